"""Pins of the oracle's tile statistics and their merge (vocabulary-tiled statistics, as the epilogue of a
tiled LM-head GEMM or a vocabulary-sharded head would hand them over).  The merged result has a plain
definition -- the statistics of the whole row (Section 3.1's entropy) -- which the oracle's row function
states and scipy pins elsewhere; here the merge is pinned to it, to scipy directly and to closed forms."""
import numpy as np
import pytest
from scipy.special import logsumexp
from scipy.stats import entropy as sp_entropy

from oracle import hola_oracle as orc
from paper_2506_18952_amd import workloads as wl


def _rows(seed, R, V, peaked=False):
    rng = np.random.default_rng(seed)
    x = rng.normal(0, 2.5, size=(R, V)).astype(np.float32)
    if peaked:
        x[np.arange(R), rng.integers(0, V, R)] += 15.0
    return x


@pytest.mark.parametrize("V,tile", [(1000, 128), (1000, 1000), (1000, 1), (4097, 512), (300, 7), (50, 64)])
@pytest.mark.parametrize("T", [1.0, 0.6])
def test_merge_equals_whole_row(V, tile, T):
    x = _rows(V + tile, 5, V, peaked=(V % 2 == 0))
    merged = orc.merge_tile_stats(orc.tile_stats(x, tile, T))
    for r in range(x.shape[0]):
        lse, H, _ = orc.row_stats(x[r], T)
        assert merged[r, 0] == pytest.approx(lse, rel=0, abs=1e-12)
        assert merged[r, 1] == pytest.approx(H, rel=0, abs=1e-11)


def test_merge_against_scipy_on_explicit_distributions():
    rng = np.random.default_rng(5)
    # tiles given directly as distributions with a mass each: the row's distribution is their mixture
    for _ in range(20):
        nt = int(rng.integers(1, 9))
        sizes = rng.integers(1, 40, nt)
        masses = rng.gamma(1.0, 1.0, nt) + 1e-3
        dists = [rng.dirichlet(np.ones(n)) for n in sizes]
        ts = np.array([[np.log(m), sp_entropy(d)] for m, d in zip(masses, dists)])[None]
        full = np.concatenate([m * d for m, d in zip(masses, dists)])
        got = orc.merge_tile_stats(ts)[0]
        assert got[0] == pytest.approx(np.log(full.sum()), abs=1e-12)
        assert got[1] == pytest.approx(sp_entropy(full / full.sum()), abs=1e-12)


def test_closed_forms():
    # n_t equal logits per tile: lse_t = c + ln n_t, H_t = ln n_t; the row is uniform over sum n_t elements
    n = np.array([3, 5, 8, 16])
    ts = np.stack([0.7 + np.log(n), np.log(n)], axis=1)[None]
    got = orc.merge_tile_stats(ts)[0]
    assert got[0] == pytest.approx(0.7 + np.log(n.sum()), abs=1e-14)
    assert got[1] == pytest.approx(np.log(n.sum()), abs=1e-14)
    # two one-element tiles with masses a and 1-a: binary entropy
    a = 0.2
    ts = np.array([[[np.log(a), 0.0], [np.log(1 - a), 0.0]]])
    got = orc.merge_tile_stats(ts)[0]
    assert got[0] == pytest.approx(0.0, abs=1e-15)
    assert got[1] == pytest.approx(-(a * np.log(a) + (1 - a) * np.log(1 - a)), abs=1e-15)
    # a single tile is the row
    assert orc.merge_tile_stats(np.array([[[1.25, 0.5]]]))[0].tolist() == [1.25, 0.5]
    # merge is invariant under permutation of the tiles and under a common shift of the lse_t
    rng = np.random.default_rng(0)
    ts = np.stack([rng.normal(0, 3, 7), rng.uniform(0, 4, 7)], axis=1)
    base = orc.merge_tile_stats(ts[None])[0]
    perm = orc.merge_tile_stats(ts[rng.permutation(7)][None])[0]
    assert perm[0] == pytest.approx(base[0], abs=1e-13) and perm[1] == pytest.approx(base[1], abs=1e-13)
    sh = ts.copy(); sh[:, 0] += 11.0
    shifted = orc.merge_tile_stats(sh[None])[0]
    assert shifted[0] == pytest.approx(base[0] + 11.0, abs=1e-12) and shifted[1] == pytest.approx(base[1], abs=1e-12)


def test_degenerate_tiles():
    inf = float("inf")
    # a tile with no finite logit carries no mass, whatever its H_t
    ts = np.array([[[-inf, float("nan")], [0.3, 1.1], [-inf, 5.0]]])
    assert orc.merge_tile_stats(ts)[0].tolist() == [0.3, 1.1]
    got = orc.merge_tile_stats(np.array([[[-inf, float("nan")]] * 3]))[0]
    assert got[0] == -inf and np.isnan(got[1])
    got = orc.merge_tile_stats(np.array([[[float("nan"), 1.0], [0.0, 1.0]]]))[0]
    assert np.isnan(got[0]) and np.isnan(got[1])
    # the tile function itself on a masked tile agrees with the row function's convention
    x = np.full((1, 8), -inf, dtype=np.float32); x[0, 5] = 1.0
    ts = orc.tile_stats(x, 4)
    assert ts[0, 0, 0] == -inf and np.isnan(ts[0, 0, 1])
    m = orc.merge_tile_stats(ts)[0]
    assert m[0] == pytest.approx(1.0) and m[1] == pytest.approx(0.0, abs=1e-15)


def test_bf16_workload_rows_merge():
    w = wl.small_case(B=2, gamma=2, V=3000, dtype="bf16", seed=11)
    rows = w.target.reshape(-1, w.V)
    merged = orc.merge_tile_stats(orc.tile_stats(rows, 512, w.temperature))
    for r in range(rows.shape[0]):
        lse, H, _ = orc.row_stats(rows[r], w.temperature)
        assert merged[r, 0] == pytest.approx(lse, abs=1e-12)
        assert merged[r, 1] == pytest.approx(H, abs=1e-11)
