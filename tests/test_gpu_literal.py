"""GPU parity of the paper-literal mode (Equation (1) without stopping) through the C ABI."""
import math

import numpy as np
import pytest
import torch

from oracle import hola_oracle as orc
from paper_2506_18952_amd import binding as hb
from paper_2506_18952_amd import workloads as wl
from parity import DEV, ENTROPY_ABS_FLOOR, MARGIN, to_dev

pytestmark = pytest.mark.gpu


def _run_gpu(w, tau, draft_len=None, seq_base=0):
    B, g, V = w.B, w.gamma, w.V
    P, D, tok = to_dev(w.target), to_dev(w.draft), to_dev(w.tokens)
    out = torch.full((B, g), -7, dtype=torch.int32, device=DEV)
    calls = torch.full((B,), -7, dtype=torch.int32, device=DEV)
    ent = torch.full((B, g), -7.0, dtype=torch.float32, device=DEV)
    ws = hb.alloc_workspace(hb.hola_workspace_bytes(B, g, V), DEV)
    dl = None if draft_len is None else to_dev(np.ascontiguousarray(draft_len, np.int32))
    rt = None if w.row_temperature is None else to_dev(w.row_temperature)
    hb.hola_verify_literal_ex(target_logits=P, draft_logits=D, draft_tokens=tok, seed=w.seed, B=B, gamma=g, V=V,
                              temperature=w.temperature, entropy_threshold=tau, out_tokens=out,
                              out_verifier_calls=calls, out_entropy=ent, workspace=ws, draft_len=dl,
                              row_temperature=rt, seq_base=seq_base)
    torch.cuda.synchronize()
    return out.cpu().numpy(), calls.cpu().numpy(), ent.cpu().numpy()


def _check(w, tau, draft_len=None, seq_base=0):
    """Every position is judged.  A token that differs from the oracle's must be the flip of a gate the oracle lists
    as near-threshold (the oracle then runs again with that gate forced to the GPU's side), or a draw whose uniform
    the oracle lists within 1e-6 of an interval end and which the GPU token's own CDF interval holds."""
    out, calls, ent = _run_gpu(w, tau, draft_len, seq_base)
    okw = dict(draft_len=draft_len, row_temperature=w.row_temperature, seq_base=seq_base)
    ref = orc.verify_literal(w.target, w.draft, w.tokens, w.seed, w.temperature, tau, **okw)
    rtol = 1e-5 if w.target.dtype == np.float32 else 2e-3
    lens = np.full(w.B, w.gamma, np.int32) if draft_len is None else np.asarray(draft_len, np.int32)
    force = np.full((w.B, w.gamma), -1, np.int8)
    listed = 0
    for b in range(w.B):
        L = int(lens[b])
        assert np.all(out[b, L:] == -1) and np.all(ent[b, L:] == -1.0)
        for t in range(L):
            h = ref.entropy64[b, t]
            err = abs(float(ent[b, t]) - h)
            assert err <= ENTROPY_ABS_FLOOR or err <= rtol * abs(h), (b, t, ent[b, t], h)
            near_gate = ref.gate_margin[b, t] < MARGIN
            listed += int(near_gate)
            if out[b, t] == ref.tokens[b, t]:
                continue
            # which side of the gate did the GPU take?  It kept the draft (oracle drew), or drew (oracle kept it).
            gpu_gated = (not ref.gate[b, t]) and out[b, t] == w.tokens[b, t]
            gpu_drew = bool(ref.gate[b, t])
            if gpu_gated or gpu_drew:
                assert near_gate, (b, t, out[b, t], ref.tokens[b, t], ref.gate_margin[b, t])
                force[b, t] = 1 if gpu_gated else 0
    flips = int((force >= 0).sum())
    if flips:
        ref = orc.verify_literal(w.target, w.draft, w.tokens, w.seed, w.temperature, tau, force_gate=force, **okw)
    tolerated = 0
    for b in range(w.B):
        Tb = float(w.temperature if w.row_temperature is None else w.row_temperature[b])
        for t in range(int(lens[b])):
            sm = ref.sample_margin[b, t]
            listed += int((not np.isnan(sm)) and sm < MARGIN)
            if out[b, t] == ref.tokens[b, t]:
                continue
            assert (not np.isnan(sm)) and sm < MARGIN, (b, t, out[b, t], ref.tokens[b, t], sm)
            iv = orc.row_interval(w.target[b, t], Tb, int(out[b, t]))
            u2 = orc.hsd_uniforms(w.seed, seq_base + b, t, 0)[1]
            assert iv is not None and iv[1] > iv[0] and iv[0] - MARGIN <= u2 <= iv[1] + MARGIN, (b, t, out[b, t], iv, u2)
            tolerated += 1
    np.testing.assert_array_equal(calls, ref.calls)
    assert flips + tolerated <= max(1, (w.B * w.gamma) // 20), (flips, tolerated)
    print(f"[parity] literal {w.name} tau={tau:.3f}: listed={listed} gate flips={flips} tolerated draws={tolerated}", flush=True)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_literal_small_and_ragged(dtype):
    w = wl.small_case(9, 5, 4099, dtype=dtype, temperature=0.9, case_id=410)
    lens = np.array([0, 1, 2, 3, 4, 5, 5, 2, 0], np.int32)
    for tau in (0.0, 0.5 * math.log(w.V), float("inf")):
        _check(w, tau)
        _check(w, tau, draft_len=lens, seq_base=(1 << 33) + 7)


def test_literal_long_drafts():
    """More drafted positions than half a wavefront (the limit is 63)."""
    w = wl.small_case(3, 63, 333, dtype="bf16", temperature=1.0, case_id=412)
    _check(w, 0.5 * math.log(w.V))


def test_literal_greedy_rows():
    w = wl.small_case(8, 4, 3001, dtype="bf16", greedy_below=4, temperature=0.7, case_id=411)
    for tau in (0.0, 0.5 * math.log(w.V)):
        _check(w, tau)


@pytest.mark.timeout(420)
def test_literal_headline_shape_subset():
    """The headline shape (V=128256 bf16, gamma=8) on 64 sequences at a threshold that splits the positions."""
    w = wl.config3(B=64)
    _check(w, w.taus[0])
    _check(w, 0.0)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_literal_aligned_rows_one_wavefront_per_draw(dtype):
    """Rows whose ends fall on the 16-byte grid, so that every verifier draw goes the quick way (one wavefront picks
    the slab from the row's partials and sweeps it alone): every position drawn (tau = 0), more draws than
    wavefronts (gamma = 20), whole slabs without mass, and a masked tail."""
    import dataclasses
    w = wl.small_case(6, 20, 16384, dtype=dtype, temperature=0.9, case_id=413)
    tgt, drf = w.target.copy(), w.draft.copy()
    neg = np.uint16(0xff80) if dtype == "bf16" else np.float32(-np.inf)
    tgt[1, :, 4096:8192] = neg                                   # a quarter of every row of sequence 1 carries no mass
    tgt[2, :, 16000:] = neg
    drf[2, :, 16000:] = neg
    w2 = dataclasses.replace(w, target=tgt, draft=drf)
    for tau in (0.0, 0.5 * math.log(w.V)):
        _check(w2, tau)


def test_literal_argument_errors():
    w = wl.small_case(2, 2, 100, case_id=412)
    P, D, tok = to_dev(w.target), to_dev(w.draft), to_dev(w.tokens)
    ws = hb.alloc_workspace(hb.hola_workspace_bytes(2, 2, 100), DEV)
    with pytest.raises(hb.HolaError):
        hb.hola_verify_literal_ex(target_logits=P, draft_logits=D, draft_tokens=tok, seed=0, B=2, gamma=2, V=100,
                                  temperature=1.0, entropy_threshold=1.0, out_tokens=None, workspace=ws)
