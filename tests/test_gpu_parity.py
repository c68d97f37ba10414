"""GPU parity: the HIP path through the C ABI against the float64 oracle, element by element, on the
named workloads (full size, in the launch configuration bench.py times) and on edge cases."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import hola_oracle as orc
from paper_2506_18952_amd import binding as hb
from paper_2506_18952_amd import workloads as wl
from parity import DEV, compare_level, run_gpu_level, to_dev

pytestmark = pytest.mark.gpu

_PATH = {"name": "auto"}


@pytest.fixture(params=["auto", "split", "fused", "split4"], autouse=True)
def kernel_path(request):
    """Every test runs with the library's own choice of kernels and with each path forced."""
    _PATH["name"] = request.param
    hb.hola_set_tuning(path={"auto": hb.PATH_AUTO, "split": hb.PATH_SPLIT, "fused": hb.PATH_FUSED,
                             "split4": hb.PATH_SPLIT4}[request.param])
    yield request.param
    hb.hola_set_tuning()


def kernel_path_name():
    return _PATH["name"]


def _report(name, rep):
    line = f"[parity] <{_PATH['name']}> {name}: {rep}"
    print(line, flush=True)
    path = os.environ.get("HOLA_PARITY_REPORT")
    if path:
        with open(path, "a") as f:
            f.write(line + "\n")


def _level(w, tau, **kw):
    gpu = run_gpu_level(w.target, w.draft, w.tokens, w.seed, w.temperature, tau,
                        row_temperature=w.row_temperature, **kw)
    okw = {k: v for k, v in kw.items() if k in ("draft_len", "seq_base", "level")}
    rep = compare_level(w.target, w.draft, w.tokens, w.seed, w.temperature, tau, gpu,
                        row_temperature=w.row_temperature, **okw)
    return gpu, rep


# ----------------------------------------------------------------------------- named workloads
def test_config1_f32_single_sequence():
    w = wl.config1()
    for tau in w.taus + [0.0, float("inf")]:
        for short in (False, True):
            gpu = run_gpu_level(w.target, w.draft, w.tokens, w.seed, w.temperature, tau, short=short)
            rep = compare_level(w.target, w.draft, w.tokens, w.seed, w.temperature, tau, gpu)
            _report(f"{w.name} tau={tau:.3f} short={short}", rep)
            assert rep.max_entropy_abs < 1e-6


def test_config2_bf16():
    w = wl.config2()
    for tau in w.taus + [0.0]:
        gpu, rep = _level(w, tau)
        _report(f"{w.name} tau={tau:.3f}", rep)
        assert rep.max_entropy_abs < 1e-6
    g2 = run_gpu_level(w.target, w.draft, w.tokens, w.seed, w.temperature, w.taus[0], short=True)
    rep = compare_level(w.target, w.draft, w.tokens, w.seed, w.temperature, w.taus[0], g2)
    _report(f"{w.name} short form", rep)


@pytest.fixture(scope="module")
def cfg3():
    return wl.config3()


def test_tuning_of_one_call_and_of_another_thread(cfg3):
    """A call's own hola_tuning decides its launch shape whatever the thread's defaults are, and a thread's
    defaults are invisible to other threads: every combination gives the decisions of the plain call."""
    import threading
    w = cfg3
    sub = slice(0, 24)
    P, D, tok = to_dev(w.target[sub]), to_dev(w.draft[sub]), to_dev(w.tokens[sub])
    B, g, V = 24, w.gamma, w.V
    tau = w.taus[0]
    base = run_gpu_level(P, D, tok, w.seed, w.temperature, tau)

    def call(tuning):
        acc = torch.full((B,), -7, dtype=torch.int32, device=DEV)
        nxt = torch.full((B,), -7, dtype=torch.int32, device=DEV)
        ent = torch.full((B, g), -7.0, dtype=torch.float32, device=DEV)
        ws = hb.alloc_workspace(hb.hola_workspace_bytes_ex(B, g, V), DEV)      # the smaller, per-call size
        hb.hola_verify_ex(target_logits=P, draft_logits=D, draft_tokens=tok, seed=w.seed, B=B, gamma=g, V=V,
                          temperature=w.temperature, entropy_threshold=tau, out_accept_len=acc, out_next_token=nxt,
                          out_entropy=ent, workspace=ws, tuning=tuning)
        torch.cuda.synchronize()
        return acc.cpu().numpy(), nxt.cpu().numpy(), ent.cpu().numpy()

    for tuning in (None, dict(path=hb.PATH_SPLIT, stats_split=4, stats_unroll=4, fused_waves=8), dict(path=hb.PATH_SPLIT4),
                   dict(path=hb.PATH_FUSED, fused_waves=8)):
        acc, nxt, ent = call(tuning)
        np.testing.assert_array_equal(acc, base.accept_len)
        np.testing.assert_array_equal(nxt, base.next_token)
        np.testing.assert_allclose(ent, base.entropy, rtol=2e-6, atol=1e-6)
    got = {}

    def other_thread():
        torch.cuda.set_device(0)
        hb.hola_set_tuning(path=hb.PATH_SPLIT4, stats_split=8)                # this thread's defaults only
        got["out"] = call(None)
    th = threading.Thread(target=other_thread)
    th.start(); th.join()
    np.testing.assert_array_equal(got["out"][0], base.accept_len)
    np.testing.assert_array_equal(got["out"][1], base.next_token)


@pytest.mark.timeout(420)
def test_config3_bf16_headline_full_size(cfg3):
    """B=256, gamma=8, V=128256 bf16, T=0.8 at three thresholds and with the gate off."""
    w = cfg3
    P, D, tok = to_dev(w.target), to_dev(w.draft), to_dev(w.tokens)
    hist = {}
    for tau in w.taus + [0.0]:
        gpu = run_gpu_level(P, D, tok, w.seed, w.temperature, tau)
        rep = compare_level(w.target, w.draft, w.tokens, w.seed, w.temperature, tau, gpu)
        _report(f"{w.name} tau={tau:.3f}", rep)
        assert rep.max_entropy_abs < 1e-6
        hist[tau] = np.bincount(gpu.accept_len, minlength=w.gamma + 1)
    print("[parity] accept-length histograms:", {f"{k:.2f}": v.tolist() for k, v in hist.items()})
    # determinism: a second run is bit-identical
    a = run_gpu_level(P, D, tok, w.seed, w.temperature, w.taus[1])
    b = run_gpu_level(P, D, tok, w.seed, w.temperature, w.taus[1])
    assert np.array_equal(a.accept_len, b.accept_len) and np.array_equal(a.next_token, b.next_token)
    assert np.array_equal(a.entropy, b.entropy)


def test_config3_launch_shapes_agree(cfg3):
    """Every launch shape of the streaming kernels gives the same decisions."""
    w = cfg3
    sub = slice(0, 32)
    P, D, tok = to_dev(w.target[sub]), to_dev(w.draft[sub]), to_dev(w.tokens[sub])
    tau = w.taus[0]
    if kernel_path_name() == "auto":
        shapes = [(hb.PATH_AUTO, 0, 0, 0)]
    elif kernel_path_name() == "split":
        shapes = [(hb.PATH_SPLIT, s, u, nw) for s, u, nw in ((1, 4, 8), (2, 2, 16), (4, 8, 8), (16, 4, 16), (1, 16, 0))]
    elif kernel_path_name() == "split4":
        shapes = [(hb.PATH_SPLIT4, s, u, 0) for s, u in ((1, 8), (2, 4), (8, 2))]
    else:
        shapes = [(hb.PATH_FUSED, 0, u, nw) for u, nw in ((2, 8), (4, 16), (8, 8), (8, 16))]
    for path, split, unroll, nw in shapes:
        hb.hola_set_tuning(split, unroll, path, nw)
        gpu = run_gpu_level(P, D, tok, w.seed, w.temperature, tau)
        rep = compare_level(w.target[sub], w.draft[sub], w.tokens[sub], w.seed, w.temperature, tau, gpu)
        _report(f"{w.name}[:32] path={path} split={split} unroll={unroll} waves={nw}", rep)
        assert rep.max_entropy_abs < 1e-6


_CFG5 = {}


def _cfg5():
    """Config 5 and the oracle's verdict on it, computed once for the four kernel paths."""
    if not _CFG5:
        w = wl.config5(B=1024)
        _CFG5["w"] = w
        _CFG5["dev"] = (to_dev(w.target), to_dev(w.draft), to_dev(w.tokens))
    return _CFG5["w"], _CFG5["dev"]


@pytest.mark.timeout(900)
def test_config5_f32_greedy_and_stochastic_rows_full_size():
    """B=1024, gamma=4, V=256000 fp32 through one call with per-row temperatures (half the rows greedy); all
    1024 sequences are compared with the oracle."""
    w, (P, D, tok) = _cfg5()
    tau = w.taus[0]
    gpu = run_gpu_level(P, D, tok, w.seed, w.temperature, tau, row_temperature=w.row_temperature)
    rep = compare_level(w.target, w.draft, w.tokens, w.seed, w.temperature, tau, gpu, row_temperature=w.row_temperature)
    _report(f"{w.name} all {w.B} sequences", rep)
    assert rep.max_entropy_abs < 1e-6
    assert rep.accept_mismatch + rep.token_mismatch <= w.B // 20
    # properties that hold at any size: greedy rows accept exactly the argmax prefix
    am = np.argmax(w.target[:8], axis=-1)
    for b in range(8):
        match = w.tokens[b] == am[b, :w.gamma]
        a = int(np.flatnonzero(~match)[0]) if (~match).any() else w.gamma
        # the gate may keep a non-argmax draft; without gate hits the prefix rule is exact
        assert gpu.accept_len[b] >= a and gpu.next_token[b] == am[b, gpu.accept_len[b]]
    assert np.all((gpu.accept_len >= 0) & (gpu.accept_len <= w.gamma))
    assert np.all((gpu.next_token >= 0) & (gpu.next_token < w.V))
    if kernel_path_name() == "split4":                           # the last of the four paths: free 19 GB
        _CFG5.clear()
        torch.cuda.empty_cache()


# ----------------------------------------------------------------------------- two-level hierarchy
def _hsd_gpu(models, tokens, seed, T, taus, row_temperature=None, survivors_only=False):
    ms = [to_dev(m) for m in models]
    n = len(ms)
    B, g, V = ms[0].shape
    L, gmax = n - 1, g + n - 2
    out_tok = torch.full((B, g + n - 1), -7, dtype=torch.int32, device=DEV)
    acc = torch.full((B,), -7, dtype=torch.int32, device=DEV)
    nxt = torch.full((B,), -7, dtype=torch.int32, device=DEV)
    ent = torch.full((L, B, gmax), -7.0, dtype=torch.float32, device=DEV)
    ws = hb.alloc_workspace(hb.hola_hsd_workspace_bytes(n, B, g, V), DEV)
    rt = None if row_temperature is None else to_dev(row_temperature)
    if survivors_only:
        hb.hola_hsd_verify_ex(ms, to_dev(tokens), seed, B, g, V, T, taus, out_tok, acc, nxt, ent, ws,
                              survivors_only=True, row_temperature=rt)
    else:
        hb.hola_hsd_verify(ms, to_dev(tokens), seed, B, g, V, T, taus, out_tok, acc, nxt, ent, ws, row_temperature=rt)
    torch.cuda.synchronize()
    return out_tok.cpu().numpy(), acc.cpu().numpy(), nxt.cpu().numpy(), ent.cpu().numpy()


def _check_hsd(models, tokens, seed, T, taus, name, survivors_only=False):
    out_tok, acc, nxt, ent = _hsd_gpu(models, tokens, seed, T, taus, survivors_only=survivors_only)
    ref = orc.hsd_verify(models, tokens, seed, T, taus, survivors_only=survivors_only)
    n = len(models)
    B, g, V = models[0].shape
    # Walk the chain level by level so that a listed near-threshold flip is judged where it happens:
    # each level of the GPU chain is compared with the oracle run on the GPU's own inputs to that level.
    cur_tok, cur_len = np.asarray(tokens, np.int32), np.full(B, g, np.int32)
    flips = 0
    for k in range(1, n):
        gk = g + k - 1
        gl = run_gpu_level(models[k], models[k - 1], cur_tok, seed, T, taus[k - 1], draft_len=cur_len, level=k - 1)
        rep = compare_level(models[k], models[k - 1], cur_tok, seed, T, taus[k - 1], gl, draft_len=cur_len, level=k - 1)
        _report(f"{name} level {k}", rep)
        flips += rep.accept_mismatch + rep.token_mismatch
        # driver (middle model's statistics reused) == stand-alone level (recomputed), up to summation order
        np.testing.assert_allclose(ent[k - 1][:, :gk], gl.entropy, rtol=2e-6, atol=1e-6)
        assert np.all(ent[k - 1][:, gk:] == -1.0)
        if k < n - 1:
            nt = np.full((B, gk + 1), -1, np.int32)
            for b in range(B):
                a = gl.accept_len[b]
                nt[b, :a] = cur_tok[b, :a]
                if not survivors_only:
                    nt[b, a] = gl.next_token[b]
            cur_tok, cur_len = nt, gl.accept_len + (0 if survivors_only else 1)
        else:
            np.testing.assert_array_equal(acc, gl.accept_len)
            np.testing.assert_array_equal(nxt, gl.next_token)
            for b in range(B):
                assert np.array_equal(out_tok[b, :cur_len[b]], cur_tok[b, :cur_len[b]])
                assert np.all(out_tok[b, cur_len[b]:] == -1)
    if flips == 0:                                                             # whole chain == oracle chain
        np.testing.assert_array_equal(acc, ref.accept_len)
        np.testing.assert_array_equal(nxt, ref.next_token)
        np.testing.assert_array_equal(out_tok, ref.tokens)
        np.testing.assert_allclose(ent, ref.entropy, rtol=2e-3, atol=2e-6)


@pytest.mark.timeout(420)
def test_config4_two_level_bf16_full_size():
    w = wl.config4()
    _check_hsd(w.models, w.tokens, w.seed, w.temperature, w.taus, w.name)


def test_three_level_small_f32():
    rng = np.random.default_rng(5)
    B, g, V = 9, 3, 1003
    base = (2 * rng.standard_normal((B, g + 3, V))).astype(np.float32)
    models = [(base[:, :g + k] + (0.9 - 0.3 * k) * rng.standard_normal((B, g + k, V))).astype(np.float32)
              for k in range(3)] + [base]
    q = np.exp(models[0].astype(np.float64))
    tok = np.array([[rng.choice(V, p=q[b, j] / q[b, j].sum()) for j in range(g)] for b in range(B)], np.int32)
    _check_hsd(models, tok, 11, 1.0, [2.0, 3.0, 4.0], "three-level small")
    _check_hsd(models, tok, 11, 1.0, [2.0, 3.0, 4.0], "three-level small, survivors only", survivors_only=True)


def test_two_level_survivors_only_bf16():
    """The other reading of the hierarchy: a level passes on only the tokens it kept."""
    w = wl.config4(B=24, V=30011, gamma=5)
    _check_hsd(w.models, w.tokens, w.seed, w.temperature, [0.0, w.taus[1]], w.name + " survivors only", survivors_only=True)


# ----------------------------------------------------------------------------- row statistics alone
def test_row_stats_entry_closed_forms_and_oracle():
    V = 128256
    rows = np.zeros((4, V), np.float32)
    rows[1] = -(2.0 ** -13) * np.arange(V)                 # geometric, exact in float32
    rows[2] = -(2.0 ** -5) * np.arange(V)
    rows[3] = np.random.default_rng(0).standard_normal(V).astype(np.float32) * 3
    for arr, rtol in ((rows, 1e-5), (wl.f32_to_bf16_bits(rows), 2e-3)):
        t = to_dev(arr)
        out = torch.zeros((4, 2), dtype=torch.float64, device=DEV)
        ws = hb.alloc_workspace(hb.hola_workspace_bytes(4, 1, V), DEV)
        hb.hola_row_stats(t, 4, V, 1.0, out, ws)
        torch.cuda.synchronize()
        o = out.cpu().numpy()
        for r in range(4):
            lse, H, _ = orc.row_stats(arr[r], 1.0)
            assert abs(o[r, 0] - lse) < 2e-6 and abs(o[r, 1] - H) <= max(rtol * abs(H), 2e-6), (r, o[r], lse, H)
        assert abs(o[0, 1] - math.log(V)) < 1e-6            # uniform logits: H = ln V
        a = 2.0 ** -13
        if arr.dtype == np.float32:
            lse_cf = math.log(-math.expm1(-a * V) / -math.expm1(-a))
            assert abs(o[1, 0] - lse_cf) < 2e-6


# ----------------------------------------------------------------------------- ragged shapes and edge cases
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,g,V", [(1, 1, 1), (3, 1, 7), (2, 2, 8), (5, 3, 1001), (4, 4, 2049), (7, 5, 4099),
                                   (3, 32, 517), (5, 33, 300), (3, 63, 517), (2, 2, 70001)])
def test_ragged_shapes(B, g, V, dtype):
    w = wl.small_case(B, g, V, dtype=dtype, temperature=0.9, case_id=200 + V % 97)
    for tau in (0.0, w.taus[0]):
        gpu, rep = _level(w, tau)
        _report(f"{w.name} tau={tau:.3f}", rep)
        assert rep.max_entropy_abs < 1e-6


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_misaligned_rows_via_leading_dimension(dtype):
    """Rows that do not start on 16-byte boundaries (ld = V + odd), target and draft misaligned differently."""
    B, g, V = 4, 3, 1237
    w = wl.small_case(B, g, V, dtype=dtype, case_id=301)
    np_dt = w.target.dtype
    ldP, ldD = V + 3, V + 5
    bufP = np.zeros((B, g + 1, ldP), np_dt)
    bufD = np.zeros((B, g, ldD), np_dt)
    bufP[:, :, :V], bufD[:, :, :V] = w.target, w.draft
    P, D, tok = to_dev(bufP), to_dev(bufD), to_dev(w.tokens)
    acc = torch.zeros(B, dtype=torch.int32, device=DEV)
    nxt = torch.zeros(B, dtype=torch.int32, device=DEV)
    ent = torch.zeros((B, g), dtype=torch.float32, device=DEV)
    ws = hb.alloc_workspace(hb.hola_workspace_bytes(B, g, V), DEV)
    from parity import GpuOut
    for tau in (0.0, w.taus[0]):
        hb.hola_verify_ex(target_logits=P, draft_logits=D, draft_tokens=tok, seed=w.seed, B=B, gamma=g, V=V,
                          temperature=w.temperature, entropy_threshold=tau, out_accept_len=acc, out_next_token=nxt,
                          out_entropy=ent, workspace=ws, target_ld=ldP, draft_ld=ldD)
        torch.cuda.synchronize()
        gpu = GpuOut(acc.cpu().numpy(), nxt.cpu().numpy(), ent.cpu().numpy())
        rep = compare_level(w.target, w.draft, w.tokens, w.seed, w.temperature, tau, gpu)
        _report(f"{w.name} misaligned tau={tau:.3f}", rep)


def test_ragged_draft_len_and_seq_base():
    w = wl.small_case(9, 5, 3001, dtype="bf16", case_id=302)
    lens = np.array([0, 1, 2, 3, 4, 5, 5, 2, 0], np.int32)
    for tau in (0.0, w.taus[0]):
        gpu, rep = _level(w, tau, draft_len=lens, seq_base=(1 << 33) + 5, level=3)
        _report(f"{w.name} ragged tau={tau:.3f}", rep)
        assert np.all(gpu.accept_len <= lens)
    # a batch row equals the single-sequence call with seq_base = b
    full = run_gpu_level(w.target, w.draft, w.tokens, w.seed, w.temperature, 0.0)
    for b in (0, 4, 8):
        one = run_gpu_level(w.target[b:b + 1], w.draft[b:b + 1], w.tokens[b:b + 1], w.seed, w.temperature, 0.0, seq_base=b)
        assert one.accept_len[0] == full.accept_len[b] and one.next_token[0] == full.next_token[b]


def test_masked_vocabulary_and_degenerate_rows():
    B, g, V = 6, 3, 2500
    w = wl.small_case(B, g, V, dtype="f32", case_id=303)
    P, D, tok = w.target.copy(), w.draft.copy(), w.tokens.copy()
    rng = np.random.default_rng(1)
    mask = rng.random(V) < 0.4                              # -inf logits: masked vocabulary
    P[:, :, mask] = -np.inf
    D[:, :, mask] = -np.inf
    for b in range(B):
        for j in range(g):
            if mask[tok[b, j]]:
                tok[b, j] = int(np.flatnonzero(~mask)[0])
    P[1, 0, tok[1, 0]] = -np.inf                            # p(x) = 0: always rejected with the gate off
    P[2, 1, :] = -np.inf                                    # a target row with no mass
    P[3, :, :] = D[3, 0, :]                                 # identical rows ...
    D[3, :, :] = D[3, 0, :]
    tok[3, 0] = V + 9                                       # ... and an out-of-range token: Z = 0 fallback
    tok[4, 1] = -2
    for tau in (0.0, 0.5 * math.log(V)):
        gpu = run_gpu_level(P, D, tok, 5, 1.0, tau)
        rep = compare_level(P, D, tok, 5, 1.0, tau, gpu)
        _report(f"masked/degenerate tau={tau:.3f}", rep)
        if tau == 0.0:
            assert gpu.accept_len[1] == 0 and gpu.accept_len[3] == 0
    gpu = run_gpu_level(P, D, tok, 5, 1.0, float("inf"))    # gate keeps everything, also p(x) = 0
    assert np.all(gpu.accept_len == g)
    # a stop row without mass gives -1
    tok2 = tok.copy()
    P2 = P.copy()
    P2[2, 0, :] = -np.inf
    g2 = run_gpu_level(P2, D, tok2, 5, 1.0, 0.0)
    r2 = orc.verify(P2, D, tok2, 5, 1.0, 0.0)
    assert g2.accept_len[2] == r2.accept_len[2] == 0 and g2.next_token[2] == r2.next_token[2] == -1


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("temperature", [0.8, 1.0, 1.3])
def test_padded_and_masked_vocabulary_on_wide_rows(dtype, temperature):
    """Rows of headline width whose last 256 entries are -inf (a padded vocabulary) and rows with 30 % of the entries
    masked: the wavefronts that meet them repeat their share with -inf left out of the sums.  Several temperatures,
    because the sign of the scale constant's low part decides whether a -inf logit spoils S as well as T."""
    B, g, V = 6, 3, 128256
    w = wl.small_case(B, g, V, dtype=dtype, temperature=temperature, case_id=305)
    P, D, tok = w.target.copy(), w.draft.copy(), w.tokens.copy()
    neg = np.uint16(0xff80) if dtype == "bf16" else np.float32(-np.inf)
    mask = np.zeros(V, bool)
    mask[V - 256:] = True
    rnd = np.random.default_rng(7).random(V) < 0.3
    for b in range(B):
        m = mask | rnd if b % 2 else mask                    # odd sequences: also 30 % masked at random
        P[b, :, m] = neg
        D[b, :, m] = neg
        ok = np.flatnonzero(~m)
        for j in range(g):
            if m[tok[b, j]]:
                tok[b, j] = int(ok[(b * 7 + j) % ok.size])
    for tau in (0.0, 0.5 * math.log(V), float("inf")):
        gpu = run_gpu_level(P, D, tok, 11, temperature, tau)
        rep = compare_level(P, D, tok, 11, temperature, tau, gpu)
        _report(f"padded/masked wide rows {dtype} T={temperature} tau={tau:.3f}", rep)
        assert rep.max_entropy_abs < 1e-6
        assert np.all((gpu.next_token < V - 256) & (gpu.next_token >= 0))


def test_huge_dynamic_range_and_identical_models():
    rng = np.random.default_rng(2)
    B, g, V = 4, 3, 5000
    P = rng.standard_normal((B, g + 1, V)).astype(np.float32)
    hot = rng.integers(0, V, (B, g + 1))
    for b in range(B):
        for j in range(g + 1):
            P[b, j, hot[b, j]] += 1e4                       # one-hot-like rows
    D = P[:, :g].copy()
    tok = hot[:, :g].astype(np.int32)
    tok[1, 1] = (tok[1, 1] + 1) % V
    for rowT in (None, np.zeros(B, np.float32)):
        gpu = run_gpu_level(P, D, tok, 1, 1.0, 0.0, row_temperature=rowT)
        rep = compare_level(P, D, tok, 1, 1.0, 0.0, gpu, row_temperature=rowT)
        _report(f"one-hot rows greedy={rowT is not None}", rep)
        assert list(gpu.accept_len) == [g, 1, g, g] and gpu.next_token[1] == hot[1, 1]
    # identical models accept everything for every seed
    w = wl.small_case(8, 4, 3000, dtype="bf16", case_id=304)
    for seed in range(5):
        gpu = run_gpu_level(w.target, w.target[:, :4].copy(), w.tokens, seed, 0.8, 0.0)
        assert np.all(gpu.accept_len == 4)


def test_greedy_rows_with_ties_small():
    B, g, V = 6, 3, 777
    w = wl.small_case(B, g, V, dtype="bf16", greedy_below=3, temperature=0.7, case_id=305)
    P = w.target.copy()
    P[0, 0, 100] = P[0, 0, 600] = np.uint16(0x4200)         # two equal maxima (32.0): lowest index wins
    tok = w.tokens.copy()
    tok[0, 0] = 100
    gpu = run_gpu_level(P, w.draft, tok, w.seed, w.temperature, 0.0, row_temperature=w.row_temperature)
    rep = compare_level(P, w.draft, tok, w.seed, w.temperature, 0.0, gpu, row_temperature=w.row_temperature)
    _report("greedy ties", rep)
    assert gpu.accept_len[0] >= 1


def test_gate_monotone_in_tau_on_gpu():
    w = wl.small_case(32, 6, 5003, dtype="bf16", case_id=306)
    P, D, tok = to_dev(w.target), to_dev(w.draft), to_dev(w.tokens)
    prev = None
    for tau in np.linspace(0, math.log(w.V) + 0.5, 12):
        gpu = run_gpu_level(P, D, tok, w.seed, w.temperature, float(tau))
        if prev is not None:
            assert np.all(gpu.accept_len >= prev)
        prev = gpu.accept_len
    assert np.all(prev == w.gamma)


def test_huge_vocabulary_falls_back_to_the_split_sampler():
    """More sampler tiles than the per-sequence kernels hold in LDS: the library must take the
    four-kernel path on its own, whatever path was asked for, and still match the oracle."""
    B, g, V = 2, 1, 2_200_000
    w = wl.small_case(B, g, V, dtype="f32", temperature=1.0, zipf_slope=None, peak_prob=0.0, case_id=307)
    for tau in (0.0, float("inf")):
        gpu, rep = _level(w, tau)
        _report(f"{w.name} tau={tau}", rep)
        assert rep.max_entropy_abs < 1e-6


def test_graph_capture_and_replay():
    """hola_verify_ex enqueues kernels only (no allocation, no host synchronisation, no memset), so a
    call can be captured in a HIP graph; every replay must reproduce the eager result."""
    w = wl.small_case(40, 4, 20011, dtype="bf16", temperature=0.8, case_id=308)
    B, g, V = w.B, w.gamma, w.V
    P, D, tok = to_dev(w.target), to_dev(w.draft), to_dev(w.tokens)
    ws = hb.alloc_workspace(hb.hola_workspace_bytes(B, g, V), DEV)
    outs = [torch.zeros(B, dtype=torch.int32, device=DEV), torch.zeros(B, dtype=torch.int32, device=DEV),
            torch.zeros((B, g), dtype=torch.float32, device=DEV)]

    def call(stream=None):
        hb.hola_verify_ex(target_logits=P, draft_logits=D, draft_tokens=tok, seed=w.seed, B=B, gamma=g, V=V,
                          temperature=w.temperature, entropy_threshold=0.0, out_accept_len=outs[0],
                          out_next_token=outs[1], out_entropy=outs[2], workspace=ws, stream=stream)

    call()
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
        call()                                              # eager work between the replays
        torch.cuda.synchronize()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("V", [2048, 16384, 100000, 131072])
def test_bonus_draw_with_mass_at_slab_boundaries(V, dtype):
    """Every draft kept (tau = +inf), so each sequence draws its bonus token from target row gamma.  With the
    split-row partials at hand that draw picks one contiguous slab of the row and re-reads only it; here most of
    the mass sits on tokens at multiples of 512 elements and their neighbours, which is where slabs begin and
    end whatever the split, and some rows hold a whole slab of -inf."""
    rng = np.random.default_rng(V % 97 + (7 if dtype == "bf16" else 0))
    B, g = 96, 2
    P = rng.normal(0, 1, (B, g + 1, V)).astype(np.float32)
    D = (P[:, :g] + rng.normal(0, 0.3, (B, g, V))).astype(np.float32)
    edges = np.arange(0, V, 512)
    for b in range(B):
        k = rng.choice(edges, size=min(6, edges.size), replace=False)
        P[b, g, k] += 9.0
        P[b, g, np.minimum(k + 511, V - 1)] += 9.0
        P[b, g, np.maximum(k - 1, 0)] += 8.5
        if b % 8 == 0:
            P[b, g, (V // 4):(V // 2)] = -np.inf                 # whole slabs without mass
        if b % 16 == 1:
            P[b, g, :] = -30.0
            P[b, g, V - 1] = 5.0                                 # all the mass on the last token
    tok = rng.integers(0, V, (B, g)).astype(np.int32)
    if dtype == "bf16":
        P, D = wl.f32_to_bf16_bits(P), wl.f32_to_bf16_bits(D)
    for seed in (3, 4):
        out = run_gpu_level(P, D, tok, seed, 1.0, float("inf"))
        assert np.all(out.accept_len == g)
        rep = compare_level(P, D, tok, seed, 1.0, float("inf"), out)
        _report(f"bonus slabs V={V} {dtype} seed={seed}", rep)
