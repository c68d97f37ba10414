"""GPU parity of the token-tree verify step (hola_verify_tree) against the oracle's walk.

Bar: kept path, accept length and next token bit-exact, except that a result may be the flip of exactly one comparison
the oracle lists as near-threshold (a gate |H - tau|, a test in the unnormalised units max(0, p - C q), or the sampling
uniform within 1e-6 of an interval end): the oracle then repeats its walk with that decision forced and the rest must
agree; no sequence is left unjudged.  Entropies as for the one-token step.  A chain must reproduce hola_verify_ex exactly."""
import math

import numpy as np
import pytest
import torch

from oracle import hola_oracle as orc
from paper_2506_18952_amd import binding as hb, workloads as wl
from parity import DEV, ENTROPY_ABS_FLOOR, MARGIN, run_gpu_level, to_dev

pytestmark = pytest.mark.gpu


def run_tree(target, draft, tok, par, seed, T, tau, n_nodes=None, level=0, seq_base=0, dev=None, want_path=True):
    P, D = dev if dev is not None else (to_dev(target), to_dev(draft))
    B, N1, V = P.shape
    N = N1 - 1
    acc = torch.full((B,), -7, dtype=torch.int32, device=DEV)
    nxt = torch.full((B,), -7, dtype=torch.int32, device=DEV)
    path = torch.full((B, N), -7, dtype=torch.int32, device=DEV) if want_path else None
    ent = torch.full((B, N), -7.0, dtype=torch.float32, device=DEV)
    ws = hb.alloc_workspace(hb.hola_tree_workspace_bytes(B, N, V), DEV)
    nn = None if n_nodes is None else to_dev(np.ascontiguousarray(n_nodes, np.int32))
    hb.hola_verify_tree(P, D, to_dev(np.ascontiguousarray(tok, np.int32)), to_dev(np.ascontiguousarray(par, np.int32)),
                        seed, B, N, V, T, tau, acc, nxt, ws, out_path=path, out_entropy=ent, n_nodes=nn, level=level,
                        seq_base=seq_base)
    torch.cuda.synchronize()
    return acc.cpu().numpy(), (path.cpu().numpy() if want_path else None), nxt.cpu().numpy(), ent.cpu().numpy()


def _first_differing_decision(pg, ag, po, ao, par, n_len):
    """Kept paths of the GPU (pg, ag nodes) and of the oracle (po, ao): the node whose decision differs first, and
    the GPU's decision about it (1 kept, 0 rejected), plus the context it hangs under."""
    d = 0
    while d < ag and d < ao and pg[d] == po[d]:
        d += 1
    ctx = int(pg[d - 1]) + 1 if d > 0 else 0
    ng = int(pg[d]) if d < ag else None
    no = int(po[d]) if d < ao else None
    assert ng is not None or no is not None
    if ng is not None and (no is None or ng < no):
        node, outcome = ng, 1                                   # the GPU kept a child the oracle rejected
    else:
        node, outcome = no, 0                                   # the GPU rejected the child the oracle kept
    kids = [k for k in range(ctx, n_len) if par[k] == ctx - 1]
    return node, outcome, ctx, (len(kids) > 0 and kids[0] == node)


def compare_tree(target, draft, tok, par, seed, T, tau, got, n_nodes=None, level=0, seq_base=0, max_tolerated=None):
    """Every sequence is judged: kept path, accept length and next token equal the oracle's, or they differ by the
    flip of exactly one decision the oracle lists as near-threshold (a node's test, or the gate of its context when
    it is the first child); the oracle then walks again with that one decision forced to the GPU's and everything
    after it must agree.  A differing next token must be listed and its own CDF interval hold the sampling uniform."""
    acc, path, nxt, ent = got
    kw = dict(n_nodes=n_nodes, level=level, seq_base=seq_base)
    ref = orc.verify_tree(target, draft, tok, par, seed, T, tau, **kw)
    B, N = tok.shape
    lens = np.full(B, N, np.int32) if n_nodes is None else np.clip(np.asarray(n_nodes, np.int32), 0, N)
    rtol = 1e-5 if np.asarray(target).dtype == np.float32 else 2e-3
    listed, max_dh = 0, 0.0
    force_node, force_out = np.full(B, -1, np.int32), np.zeros(B, np.int32)
    for b in range(B):
        for c in range(N):
            if ref.entropy[b, c] < 0:
                assert ent[b, c] == -1.0, (b, c, ent[b, c])
                continue
            h, hg = ref.entropy64[b, c], float(ent[b, c])
            err = abs(hg - h)
            max_dh = max(max_dh, err)
            assert err <= max(rtol * abs(h), ENTROPY_ABS_FLOOR) and err < 1e-6, (b, c, hg, h)
        m = np.r_[ref.gate_margin[b], ref.ratio_margin[b], ref.sample_margin[b]]
        if np.nanmin(np.r_[m, np.inf]) < MARGIN:
            listed += 1
        a = int(acc[b])
        assert 0 <= a <= N and np.all(path[b, a:] == -1) and np.all(path[b, :a] >= 0), (b, a, path[b])
        if a == ref.accept_len[b] and np.array_equal(path[b], ref.path[b]):
            continue
        node, outcome, ctx, is_first = _first_differing_decision(path[b], a, ref.path[b], int(ref.accept_len[b]),
                                                                 par[b], int(lens[b]))
        mg = ref.ratio_margin[b, node]
        mg = np.inf if np.isnan(mg) else mg
        if is_first and not np.isnan(ref.gate_margin[b, ctx]):
            mg = min(mg, ref.gate_margin[b, ctx])
        assert mg < MARGIN, (f"seq {b}: path gpu {path[b, :a].tolist()} vs oracle {ref.path[b, :ref.accept_len[b]].tolist()}; "
                             f"node {node} under context {ctx} decides, margin {mg:.3e} (not listed near-threshold)")
        force_node[b], force_out[b] = node, outcome
    tolerated = int((force_node >= 0).sum())
    ref_acc, ref_path = ref.accept_len.copy(), ref.path.copy()
    ref_tok, ref_sm = ref.next_token.copy(), ref.sample_margin.copy()
    if tolerated:
        ref2 = orc.verify_tree(target, draft, tok, par, seed, T, tau, force_node=force_node, force_outcome=force_out, **kw)
        sel = force_node >= 0
        ref_acc[sel], ref_path[sel] = ref2.accept_len[sel], ref2.path[sel]
        ref_tok[sel], ref_sm[sel] = ref2.next_token[sel], ref2.sample_margin[sel]
    np.testing.assert_array_equal(acc, ref_acc)
    np.testing.assert_array_equal(path, ref_path)
    differ = np.flatnonzero(nxt != ref_tok)
    if differ.size:
        for b in differ:
            assert ref_sm[b] < MARGIN, f"seq {b}: next_token gpu {nxt[b]} vs oracle {ref_tok[b]}, margin {ref_sm[b]:.3e} (not listed)"
        probe = np.full(B, -1, np.int32)
        probe[differ] = nxt[differ]
        ref3 = orc.verify_tree(target, draft, tok, par, seed, T, tau, force_node=force_node, force_outcome=force_out,
                               probe_token=probe, **kw)
        for b in differ:
            lo, hi = ref3.probe_lo[b], ref3.probe_hi[b]
            ctx = int(path[b, acc[b] - 1]) + 1 if acc[b] > 0 else 0
            u2 = orc.hsd_uniforms(seed, seq_base + int(b), ctx, level)[1]
            assert hi > lo and lo - MARGIN <= u2 <= hi + MARGIN, f"seq {b}: gpu token {nxt[b]} interval ({lo}, {hi}) does not hold u'={u2}"
            if force_node[b] < 0:
                tolerated += 1
    if max_tolerated is None:
        max_tolerated = max(1, B // 20)
    assert tolerated <= max_tolerated, f"{tolerated} of {B} sequences differ from the oracle by a listed flip"
    return listed, max_dh, ref


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_chain_reproduces_the_one_token_step(dtype):
    w = wl.small_case(40, 6, 5003, dtype=dtype, temperature=0.9, case_id=41)
    par = np.tile(np.arange(-1, w.gamma - 1, dtype=np.int32), (w.B, 1))
    dl = np.array([b % (w.gamma + 1) for b in range(w.B)], np.int32)
    for tau in (-1.0, w.taus[0]):
        for kw in ({}, {"level": 2, "seq_base": 1 << 34}):
            one = run_gpu_level(w.target, w.draft, w.tokens, w.seed, w.temperature, tau, draft_len=dl, **kw)
            acc, path, nxt, ent = run_tree(w.target, w.draft, w.tokens, par, w.seed, w.temperature, tau, n_nodes=dl, **kw)
            np.testing.assert_array_equal(acc, one.accept_len)
            np.testing.assert_array_equal(nxt, one.next_token)
            np.testing.assert_array_equal(ent, one.entropy)
            for b in range(w.B):
                assert path[b, :acc[b]].tolist() == list(range(acc[b])) and np.all(path[b, acc[b]:] == -1)
    assert len(set(acc.tolist())) > 2


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("widths,V", [([3], 1001), ([2, 4, 4], 3001), ([4, 3, 2, 1, 1], 9001), ([1, 2, 1, 3], 2049),
                                      ([4, 4, 4, 4, 4, 4, 4, 4], 1500), ([8, 8, 8, 8, 8, 8, 8, 7], 1200)])
def test_small_trees(dtype, widths, V):
    w = wl.tree_case(16, widths, V, dtype=dtype, temperature=0.8, draft_sigma=1.0, case_id=750 + len(widths))
    nn = np.array([w.N - (b % 3) for b in range(w.B)], np.int32)
    for tau in (-1.0, w.tau):
        got = run_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, w.temperature, tau, n_nodes=nn)
        listed, dh, ref = compare_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, w.temperature, tau, got,
                                       n_nodes=nn)
        print(f"[parity] {w.name} tau={tau:.2f}: listed={listed} max|dH|={dh:.2e} "
              f"depth hist {np.bincount(got[0], minlength=len(widths) + 1).tolist()}", flush=True)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_many_rejected_candidates_at_one_context(dtype):
    """A drafter far from the verifier: most candidates are rejected, so the later tests and the final draw run on
    max(0, p - C q) with C well above 1."""
    w = wl.tree_case(48, [12, 6], 4001, dtype=dtype, temperature=1.0, draft_sigma=3.0, peak_prob=0.0, case_id=760)
    got = run_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, w.temperature, -1.0)
    listed, dh, ref = compare_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, w.temperature, -1.0, got)
    tested = (~np.isnan(ref.ratio_margin)).sum(axis=1)
    assert (tested >= 6).sum() >= 5 and (ref.accept_len == 0).sum() >= 3
    print(f"[parity] {w.name}: listed={listed} tests per sequence {np.bincount(tested).tolist()}", flush=True)


def test_duplicate_and_out_of_range_candidates():
    w = wl.tree_case(24, [4, 4], 2001, dtype="bf16", temperature=1.0, draft_sigma=1.5, case_id=770)
    tok = w.node_token.copy()
    tok[:, 1] = tok[:, 0]                                       # the same token offered twice
    tok[::3, 2] = -1
    tok[1::3, 3] = w.V
    got = run_tree(w.target, w.draft, tok, w.node_parent, w.seed, 1.0, -1.0)
    compare_tree(w.target, w.draft, tok, w.node_parent, w.seed, 1.0, -1.0, got)


def test_a_node_with_an_invalid_parent_is_ignored():
    w = wl.tree_case(12, [3, 3], 1001, dtype="f32", case_id=771)
    par = w.node_parent.copy()
    par[:, -1] = w.N - 1                                        # the last node names itself: no one's child
    got = run_tree(w.target, w.draft, w.node_token, par, w.seed, 1.0, -1.0)
    nn = np.full(w.B, w.N - 1, np.int32)                        # the oracle refuses such a parent: it gets one node fewer
    compare_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, 1.0, -1.0, got, n_nodes=nn)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("V", [1, 7, 64, 70001])
def test_edge_shapes(dtype, V):
    w = wl.tree_case(5, [2, 3], V, dtype=dtype, case_id=780 + V % 13)
    for nn in (None, np.zeros(w.B, np.int32), np.array([0, 1, 2, 4, 5], np.int32)):
        got = run_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, 1.0, 0.3 * math.log(max(V, 2)), n_nodes=nn)
        compare_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, 1.0, 0.3 * math.log(max(V, 2)), got,
                     n_nodes=nn)


def test_gate_everywhere_keeps_the_first_children():
    w = wl.tree_case(10, [3, 2, 2, 2], 3001, dtype="bf16", case_id=790)
    acc, path, nxt, ent = run_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, 1.0, 1e30)
    ref = orc.verify_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, 1.0, 1e30)
    np.testing.assert_array_equal(acc, ref.accept_len)
    np.testing.assert_array_equal(path, ref.path)
    assert np.all(acc == 4)


def test_without_path_output_and_determinism():
    w = wl.tree_case(20, [4, 2, 2], 6001, dtype="bf16", case_id=791)
    a = run_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, 0.7, w.tau)
    b = run_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, 0.7, w.tau, want_path=False)
    c = run_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, 0.7, w.tau)
    for x, y in ((a[0], b[0]), (a[2], b[2]), (a[0], c[0]), (a[1], c[1]), (a[2], c[2]), (a[3], c[3])):
        np.testing.assert_array_equal(x, y)


def test_unsupported_and_invalid_arguments():
    w = wl.tree_case(3, [2], 101, case_id=792)
    P, D = to_dev(w.target), to_dev(w.draft)
    tok, par = to_dev(w.node_token), to_dev(w.node_parent)
    acc = torch.zeros(3, dtype=torch.int32, device=DEV)
    nxt = torch.zeros(3, dtype=torch.int32, device=DEV)
    ws = hb.alloc_workspace(hb.hola_tree_workspace_bytes(3, w.N, w.V), DEV)
    with pytest.raises(hb.HolaError):                           # greedy rows are not taken
        hb.hola_verify_tree(P, D, tok, par, 1, 3, w.N, w.V, 0.0, 0.0, acc, nxt, ws)
    with pytest.raises(hb.HolaError):                           # workspace too small
        hb.hola_verify_tree(P, D, tok, par, 1, 3, w.N, w.V, 1.0, 0.0, acc, nxt, ws[:256])
    with pytest.raises(hb.HolaError):
        hb.hola_verify_tree(P, D, tok, par, 1, 3, 64, w.V, 1.0, 0.0, acc, nxt, ws)
    assert hb.hola_tree_workspace_bytes(3, 64, 101) == 0 and hb.hola_tree_workspace_bytes(3, 0, 101) == 0


@pytest.mark.timeout(600)
def test_headline_vocabulary_tree_against_the_oracle():
    """128256-wide bf16 rows, 64 sequences of a 16-node tree in one call; the oracle walks every one of them."""
    w = wl.tree_case(64, [4, 4, 4, 2, 2], 128256, dtype="bf16", temperature=0.8, zipf_slope=1.2, peak_prob=0.3, case_id=795)
    dev = (to_dev(w.target), to_dev(w.draft))
    for tau in (-1.0, 0.25 * math.log(w.V)):
        got = run_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, w.temperature, tau, dev=dev)
        acc, path, nxt, ent = got
        listed, dh, ref = compare_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, w.temperature, tau, got)
        assert np.all((nxt >= 0) & (nxt < w.V)) and np.all((acc >= 0) & (acc <= 5))
        print(f"[parity] {w.name} tau={tau:.2f}: all {w.B} sequences judged, listed={listed}, max|dH|={dh:.2e}, "
              f"depth hist {np.bincount(acc, minlength=6).tolist()}", flush=True)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_random_topologies_per_sequence(dtype, seed):
    """Every sequence its own random tree (chains, stars, bushes), ragged node counts, shapes off the tile grid."""
    rng = np.random.default_rng(900 + seed)
    N = int(rng.integers(1, 64))
    V = int(rng.choice([37, 1000, 4097, 12289]))
    B = int(rng.integers(1, 40))
    w = wl.tree_case(B, [N], V, dtype=dtype, temperature=float(rng.choice([0.6, 1.0, 1.7])),
                     draft_sigma=float(rng.choice([0.5, 1.5])), case_id=800 + seed, random_topology=True)
    nn = rng.integers(0, N + 1, B).astype(np.int32)
    for tau in (-1.0, 0.4 * math.log(V)):
        got = run_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, w.temperature, tau, n_nodes=nn,
                       level=seed, seq_base=seed * 1000)
        listed, dh, ref = compare_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, w.temperature, tau, got,
                                       n_nodes=nn, level=seed, seq_base=seed * 1000)
        print(f"[parity] random trees B={B} N={N} V={V} {dtype} tau={tau:.2f}: listed={listed} "
              f"depth hist {np.bincount(got[0]).tolist()}", flush=True)


def test_tree_call_in_a_hip_graph():
    """The three launches of a call captured once and replayed with the program's own work in between."""
    w = wl.tree_case(12, [3, 3, 2], 5001, dtype="bf16", case_id=796)
    P, D = to_dev(w.target), to_dev(w.draft)
    tok, par = to_dev(w.node_token), to_dev(w.node_parent)
    B, N, V = w.B, w.N, w.V
    acc = torch.full((B,), -7, dtype=torch.int32, device=DEV)
    nxt = torch.full((B,), -7, dtype=torch.int32, device=DEV)
    path = torch.full((B, N), -7, dtype=torch.int32, device=DEV)
    ws = hb.alloc_workspace(hb.hola_tree_workspace_bytes(B, N, V), DEV)
    eager = run_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, 1.0, w.tau, dev=(P, D))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            hb.hola_verify_tree(P, D, tok, par, w.seed, B, N, V, 1.0, w.tau, acc, nxt, ws, out_path=path, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    for _ in range(3):
        acc.fill_(-7); nxt.fill_(-7); path.fill_(-7)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        np.testing.assert_array_equal(acc.cpu().numpy(), eager[0])
        np.testing.assert_array_equal(path.cpu().numpy(), eager[1])
        np.testing.assert_array_equal(nxt.cpu().numpy(), eager[2])


def test_more_sequences_than_compute_units_and_strided_rows():
    """Beyond one sequence per compute unit the tail kernel runs 8 wavefronts per workgroup; rows may sit in wider
    buffers (row strides above V, rows not 16-byte aligned)."""
    w = wl.tree_case(2100, [3, 2, 2], 1003, dtype="bf16", temperature=0.9, draft_sigma=1.2, case_id=797)
    got = run_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, w.temperature, -1.0)
    compare_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, w.temperature, -1.0, got)
    hb.hola_set_tuning(fused_waves=8)
    try:
        got8 = run_tree(w.target[:40], w.draft[:40], w.node_token[:40], w.node_parent[:40], w.seed, w.temperature, -1.0)
    finally:
        hb.hola_set_tuning()
    for x, y in zip(got, got8):
        np.testing.assert_array_equal(x[:40], y)
    # the same rows inside buffers with a stride of V + 5 elements
    B, N, V = 40, w.N, w.V
    ld = V + 5
    Pw = np.zeros((B, N + 1, ld), np.uint16)
    Dw = np.zeros((B, N, ld), np.uint16)
    Pw[:, :, :V], Dw[:, :, :V] = w.target[:B], w.draft[:B]
    Pw[:, :, V:], Dw[:, :, V:] = 0x7f80, 0x7f80                 # +inf beside the rows: must never be read as logits
    P, D = to_dev(Pw), to_dev(Dw)
    acc = torch.full((B,), -7, dtype=torch.int32, device=DEV)
    nxt = torch.full((B,), -7, dtype=torch.int32, device=DEV)
    path = torch.full((B, N), -7, dtype=torch.int32, device=DEV)
    ent = torch.full((B, N), -7.0, dtype=torch.float32, device=DEV)
    ws = hb.alloc_workspace(hb.hola_tree_workspace_bytes(B, N, V), DEV)
    hb.hola_verify_tree(P, D, to_dev(w.node_token[:B]), to_dev(w.node_parent[:B]), w.seed, B, N, V, w.temperature, -1.0,
                        acc, nxt, ws, out_path=path, out_entropy=ent, target_ld=ld, draft_ld=ld)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(acc.cpu().numpy(), got[0][:B])
    np.testing.assert_array_equal(path.cpu().numpy(), got[1][:B])
    np.testing.assert_array_equal(nxt.cpu().numpy(), got[2][:B])
    np.testing.assert_allclose(ent.cpu().numpy(), got[3][:B], rtol=1e-5, atol=1e-6)


def test_empty_batch_and_single_node():
    w = wl.tree_case(2, [1], 129, dtype="f32", case_id=798)
    P, D = to_dev(w.target), to_dev(w.draft)
    acc = torch.full((2,), -7, dtype=torch.int32, device=DEV)
    nxt = torch.full((2,), -7, dtype=torch.int32, device=DEV)
    ws = hb.alloc_workspace(hb.hola_tree_workspace_bytes(2, 1, w.V), DEV)
    hb.hola_verify_tree(P, D, to_dev(w.node_token), to_dev(w.node_parent), w.seed, 0, 1, w.V, 1.0, 0.0, acc, nxt, ws)
    torch.cuda.synchronize()
    assert np.all(acc.cpu().numpy() == -7) and np.all(nxt.cpu().numpy() == -7)     # B = 0: nothing is written
    got = run_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, 1.0, 0.0)
    compare_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, 1.0, 0.0, got)
    one = run_gpu_level(w.target, w.draft, w.node_token, w.seed, 1.0, 0.0)          # one node = one drafted position
    np.testing.assert_array_equal(got[0], one.accept_len)
    np.testing.assert_array_equal(got[2], one.next_token)


@pytest.mark.parametrize("split", [1, 4, 16])
def test_statistics_split_does_not_change_the_walk(split):
    """Rows cut into 1, 4 or 16 segments by the statistics pass: other partial sums, the same decisions."""
    w = wl.tree_case(10, [3, 3, 2], 70001, dtype="bf16", temperature=0.8, case_id=799)
    base = run_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, w.temperature, w.tau)
    compare_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, w.temperature, w.tau, base)
    hb.hola_set_tuning(stats_split=split)
    try:
        got = run_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, w.temperature, w.tau)
    finally:
        hb.hola_set_tuning()
    compare_tree(w.target, w.draft, w.node_token, w.node_parent, w.seed, w.temperature, w.tau, got)
    np.testing.assert_allclose(got[3], base[3], rtol=1e-6, atol=1e-6)
