"""GPU parity on randomly drawn small shapes: batch, draft length, vocabulary (with an eye on chunk, tile, slab and
segment boundaries), logit type, temperature, threshold, ragged draft lengths, and the four filter settings.  Each
seed fixes one case; the bar is the one of the other parity tests."""
import math

import numpy as np
import pytest

from paper_2506_18952_amd import binding as hb, workloads as wl
from parity import compare_level, run_gpu_level
from test_gpu_filtered import compare_filtered, run_filtered

pytestmark = pytest.mark.gpu

_EDGE_V = [1, 2, 7, 8, 9, 63, 64, 65, 255, 256, 257, 511, 512, 513, 767, 768, 769, 1023, 1024, 1025, 2047, 2048, 2049,
           4095, 4096, 4097, 8191, 8192, 8193, 16383, 16384, 16385, 16392, 32767, 32768, 32776, 40001]


@pytest.mark.parametrize("seed", range(96))
def test_random_case(seed):
    rng = np.random.default_rng(1000 + seed)
    B = int(rng.integers(1, 10))
    g = int(rng.integers(1, 7))
    V = int(rng.choice(_EDGE_V)) if rng.random() < 0.7 else int(rng.integers(1, 40000))
    dtype = "bf16" if rng.random() < 0.5 else "f32"
    T = float(rng.choice([0.3, 0.7, 1.0, 1.6]))
    w = wl.small_case(B, g, V, dtype=dtype, temperature=T, case_id=2000 + seed, seed=50 + seed,
                      peak_prob=float(rng.choice([0.0, 0.2, 0.6])))
    dl = rng.integers(0, g + 1, B).astype(np.int32) if rng.random() < 0.5 else None
    tau = float(rng.choice([-1.0, 0.0, 0.3, 0.6, 2.0])) * math.log(max(V, 2))
    kind = seed % 4
    if kind == 0:
        out = run_gpu_level(w.target, w.draft, w.tokens, w.seed, T, tau, draft_len=dl)
        rep = compare_level(w.target, w.draft, w.tokens, w.seed, T, tau, out, draft_len=dl)
        print(f"[parity] random seed={seed} B={B} g={g} V={V} {dtype} T={T} tau={tau:.2f}: {rep}", flush=True)
        return
    top_k = int(rng.choice([1, 2, 5, 40, 64, 100])) if kind in (1, 3) else 0
    top_p = float(rng.choice([0.1, 0.5, 0.9, 0.99])) if kind in (2, 3) else 0.0
    for path in (0, 1):
        hb.hola_set_tuning(filter_path=path)
        try:
            got = run_filtered(w.target, w.draft, w.tokens, w.seed, T, tau, top_k, top_p, draft_len=dl)
            compare_filtered(w.target, w.draft, w.tokens, w.seed, T, tau, top_k, top_p, got, draft_len=dl)
        finally:
            hb.hola_set_tuning()
