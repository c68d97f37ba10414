"""GPU: a sequence's tail shared by two or four workgroups (hola_tuning.tail_split) gives, bit for bit, what one
workgroup gives, whatever the workspace held before, call after call and under HIP-graph replay; and what it gives
meets the oracle."""
import numpy as np
import pytest
import torch

from paper_2506_18952_amd import binding as hb
from paper_2506_18952_amd import workloads as wl
from parity import DEV, compare_level, GpuOut, to_dev

pytestmark = pytest.mark.gpu


def _dirty_workspace(nbytes, pattern):
    """A workspace with contents of some earlier life: all ones, small counters, or random bytes."""
    if pattern == "ones":
        return torch.full((nbytes,), 0xFF, dtype=torch.uint8, device=DEV)
    if pattern == "counters":                 # every 64-bit word reads as 1: a count without this call's tag
        w = torch.zeros(nbytes // 8, dtype=torch.int64, device=DEV) + 1
        return w.view(torch.uint8)
    g = torch.Generator(device=DEV)
    g.manual_seed(1234)
    return torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device=DEV, generator=g)


def _call(P, D, tok, w, tau, split, ws, draft_len=None, row_temperature=None, stream=None, outs=None):
    B, g1, V = P.shape
    g = g1 - 1
    if outs is None:
        outs = (torch.full((B,), -7, dtype=torch.int32, device=DEV), torch.full((B,), -7, dtype=torch.int32, device=DEV),
                torch.full((B, g), -7.0, dtype=torch.float32, device=DEV))
    hb.hola_verify_ex(target_logits=P, draft_logits=D, draft_tokens=tok, seed=w.seed, B=B, gamma=g, V=V,
                      temperature=w.temperature, entropy_threshold=tau, out_accept_len=outs[0], out_next_token=outs[1],
                      out_entropy=outs[2], workspace=ws, draft_len=draft_len, row_temperature=row_temperature,
                      tuning=dict(path=hb.PATH_SPLIT, tail_split=split), stream=stream)
    return outs


def _host(outs):
    torch.cuda.synchronize()
    return GpuOut(outs[0].cpu().numpy(), outs[1].cpu().numpy(), outs[2].cpu().numpy())


@pytest.mark.parametrize("pattern", ["ones", "counters", "random"])
@pytest.mark.parametrize("B", [5, 61, 128])
def test_shared_tail_equals_single_workgroup_bf16(B, pattern):
    """Headline rows (V=128256, bf16, 256 KB each) on few sequences: 2, 4 and 8 workgroups per sequence against 1, on a
    workspace that is never cleared, twice in a row."""
    w = wl.config3(B=B)
    P, D, tok = to_dev(w.target), to_dev(w.draft), to_dev(w.tokens)
    nbytes = hb.hola_workspace_bytes(B, w.gamma, w.V)
    for tau in (w.taus[0], 0.0):
        base = _host(_call(P, D, tok, w, tau, 1, hb.alloc_workspace(nbytes, DEV)))
        if pattern == "ones" and B <= 61:
            rep = compare_level(w.target, w.draft, w.tokens, w.seed, w.temperature, tau, base)
            print(f"[parity] tail_split base B={B} tau={tau:.3f}: {rep}", flush=True)
        assert (base.accept_len < w.gamma).any() or tau == 0.0
        for split in (2, 4, 8):
            ws = _dirty_workspace(nbytes, pattern)
            for rep_i in range(2):
                got = _host(_call(P, D, tok, w, tau, split, ws))
                np.testing.assert_array_equal(got.accept_len, base.accept_len, err_msg=f"split {split} call {rep_i}")
                np.testing.assert_array_equal(got.next_token, base.next_token, err_msg=f"split {split} call {rep_i}")
                np.testing.assert_array_equal(got.entropy, base.entropy)


def test_shared_tail_f32_short_drafts_and_row_temperatures():
    """fp32 rows of V=151936 with ragged draft lengths (0 included) and per-sequence temperatures (greedy ones
    included): the shared tail against one workgroup and against the oracle."""
    w = wl.small_case(40, 6, 151936, dtype="f32", temperature=1.0, case_id=978)
    B, g = w.B, w.gamma
    rng = np.random.default_rng(77)
    dl = rng.integers(0, g + 1, size=B).astype(np.int32)
    dl[:3] = (0, g, 1)
    rt = rng.choice(np.array([0.0, 0.6, 1.0, 1.3], np.float32), size=B).astype(np.float32)
    P, D, tok = to_dev(w.target), to_dev(w.draft), to_dev(w.tokens)
    dld, rtd = to_dev(dl), to_dev(rt)
    nbytes = hb.hola_workspace_bytes(B, g, w.V)
    tau = w.taus[0]
    base = _host(_call(P, D, tok, w, tau, 1, hb.alloc_workspace(nbytes, DEV), dld, rtd))
    rep = compare_level(w.target, w.draft, w.tokens, w.seed, w.temperature, tau, base, draft_len=dl, row_temperature=rt)
    print(f"[parity] tail_split f32 ragged: {rep}", flush=True)
    for split in (0, 2, 4, 8):
        ws = _dirty_workspace(nbytes, "random")
        for _ in range(2):
            got = _host(_call(P, D, tok, w, tau, split, ws, dld, rtd))
            np.testing.assert_array_equal(got.accept_len, base.accept_len)
            np.testing.assert_array_equal(got.next_token, base.next_token)
            np.testing.assert_array_equal(got.entropy, base.entropy)


def test_shared_tail_is_refused_where_it_cannot_run():
    """More workgroups than compute units, or rows of too few tiles: the call runs with one workgroup per sequence
    and gives the same result (the setting is a wish, not an error)."""
    w = wl.small_case(300, 3, 3000, dtype="bf16", temperature=0.9, case_id=977)
    P, D, tok = to_dev(w.target), to_dev(w.draft), to_dev(w.tokens)
    nbytes = hb.hola_workspace_bytes(w.B, w.gamma, w.V)
    base = _host(_call(P, D, tok, w, 0.0, 1, hb.alloc_workspace(nbytes, DEV)))
    got = _host(_call(P, D, tok, w, 0.0, 4, _dirty_workspace(nbytes, "ones")))
    np.testing.assert_array_equal(got.accept_len, base.accept_len)
    np.testing.assert_array_equal(got.next_token, base.next_token)


def test_shared_tail_in_a_hip_graph():
    """The tickets are left as a replay needs them: every replay of a captured call with a shared tail reproduces the
    eager result, with eager calls on the same workspace in between."""
    w = wl.config3(B=32)
    B, g, V = w.B, w.gamma, w.V
    P, D, tok = to_dev(w.target), to_dev(w.draft), to_dev(w.tokens)
    nbytes = hb.hola_workspace_bytes(B, g, V)
    ws = _dirty_workspace(nbytes, "random")
    tau = w.taus[1]
    base = _host(_call(P, D, tok, w, tau, 1, hb.alloc_workspace(nbytes, DEV)))
    outs = (torch.zeros(B, dtype=torch.int32, device=DEV), torch.zeros(B, dtype=torch.int32, device=DEV),
            torch.zeros((B, g), dtype=torch.float32, device=DEV))
    _call(P, D, tok, w, tau, 4, ws, outs=outs)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            _call(P, D, tok, w, tau, 4, ws, stream=side, outs=outs)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(4):
        for o in outs:
            o.fill_(-5)
        torch.cuda.synchronize()
        graph.replay()
        got = _host(outs)
        np.testing.assert_array_equal(got.accept_len, base.accept_len, err_msg=f"replay {rep}")
        np.testing.assert_array_equal(got.next_token, base.next_token, err_msg=f"replay {rep}")
        np.testing.assert_array_equal(got.entropy, base.entropy)
        _call(P, D, tok, w, tau, 2, ws)                        # eager work on the same workspace between the replays
        torch.cuda.synchronize()


def test_two_batches_in_flight_on_two_streams():
    """Two independent batches, each with its own workspace and outputs, issued alternately on two streams (their
    kernels overlap on the chip, shared tails and their tickets included): every call gives what it gives alone."""
    w = wl.config3(B=24)
    B, g, V = w.B, w.gamma, w.V
    nbytes = hb.hola_workspace_bytes(B, g, V)
    n_calls = 12
    sets = []
    for k in range(2):
        sub = slice(0, B) if k == 0 else slice(None, None, -1)     # the second batch: the same sequences in reverse order
        sets.append(dict(P=to_dev(np.ascontiguousarray(w.target[sub])), D=to_dev(np.ascontiguousarray(w.draft[sub])),
                         tok=to_dev(np.ascontiguousarray(w.tokens[sub])), ws=_dirty_workspace(nbytes, "random"),
                         stream=torch.cuda.Stream()))

    def call(k, i, stream, outs):
        s = sets[k]
        hb.hola_verify_ex(target_logits=s["P"], draft_logits=s["D"], draft_tokens=s["tok"], seed=w.seed + i, B=B, gamma=g, V=V,
                          temperature=w.temperature, entropy_threshold=w.taus[0], out_accept_len=outs[0], out_next_token=outs[1],
                          out_entropy=outs[2], workspace=s["ws"], stream=stream)

    def fresh():
        return (torch.full((B,), -7, dtype=torch.int32, device=DEV), torch.full((B,), -7, dtype=torch.int32, device=DEV),
                torch.full((B, g), -7.0, dtype=torch.float32, device=DEV))

    alone = {}
    for k in range(2):
        for i in range(n_calls):
            o = fresh()
            call(k, i, torch.cuda.current_stream(), o)
            alone[(k, i)] = _host(o)
    torch.cuda.synchronize()
    together = {}
    for i in range(n_calls):
        for k in range(2):
            o = fresh()
            call(k, i, sets[k]["stream"], o)
            together[(k, i)] = o
    torch.cuda.synchronize()
    rejected = 0
    for key, o in together.items():
        got, ref = _host(o), alone[key]
        np.testing.assert_array_equal(got.accept_len, ref.accept_len, err_msg=str(key))
        np.testing.assert_array_equal(got.next_token, ref.next_token, err_msg=str(key))
        np.testing.assert_array_equal(got.entropy, ref.entropy)
        rejected += int((ref.accept_len < g).sum())
    assert rejected > 0                                           # residual draws, hence shared sweeps, took part
