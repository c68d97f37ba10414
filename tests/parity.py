"""Helpers of the GPU parity tests: run one verify level through the C ABI, run the oracle on the
same inputs, and compare under the parity bar:

  * accept lengths and next tokens bit-exact, except where the oracle itself lists the deciding
    comparison as near-threshold (margin < 1e-6): a gate |H - tau|, a ratio |u - p_x/q_x|, or a
    sample whose uniform lies within 1e-6 of the chosen CDF interval's end.  A GPU result that
    differs is tolerated only if it is the outcome of flipping exactly that listed decision;
  * entropies: relative error <= 1e-5 for fp32 logits, <= 2e-3 for bf16 logits (the inputs are
    bit-identical on both sides, so the observed error is far smaller; it is reported).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

from oracle import hola_oracle as orc
from paper_2506_18952_amd import binding as hb

MARGIN = 1e-6
# A relative bar is ill-posed as H -> 0 (a nearly one-hot row): the kernel's terms 2^y are fp32, so ln S
# and with it H carry an absolute error of a few fp32 unit roundoffs of 1.0 whatever H is.  Differences
# below 4 * 2^-24 are therefore accepted outright; above it the relative bar applies.
ENTROPY_ABS_FLOOR = 4 * 2.0 ** -24
DEV = "cuda:0"


def to_dev(a: Optional[np.ndarray]):
    if a is None:
        return None
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(DEV)
    return torch.from_numpy(a).to(DEV)


@dataclass
class GpuOut:
    accept_len: np.ndarray
    next_token: np.ndarray
    entropy: np.ndarray
    target_stats: Optional[np.ndarray] = None


def run_gpu_level(target, draft, tokens, seed, temperature, tau, *, draft_len=None, row_temperature=None,
                  seq_base=0, level=0, draft_stats_in=None, target_stats_in=None, want_target_stats=False,
                  short=False, dev_inputs=None) -> GpuOut:
    """One level through the C ABI.  `target`/`draft` are numpy (uint16 = bf16 bits) or device tensors."""
    P = target if torch.is_tensor(target) else to_dev(target)
    D = draft if torch.is_tensor(draft) else to_dev(draft)
    B, g1, V = P.shape
    g = g1 - 1
    tok = tokens if torch.is_tensor(tokens) else to_dev(np.ascontiguousarray(tokens, np.int32))
    acc = torch.full((B,), -7, dtype=torch.int32, device=DEV)
    nxt = torch.full((B,), -7, dtype=torch.int32, device=DEV)
    ent = torch.full((B, g), -7.0, dtype=torch.float32, device=DEV)
    if short:
        fn = hb.hola_verify_f32 if P.dtype == torch.float32 else hb.hola_verify_bf16
        fn(P, D, tok, seed, B, g, V, temperature, tau, acc, nxt, ent)
        tstats = None
    else:
        ws = hb.alloc_workspace(hb.hola_workspace_bytes(B, g, V), DEV)
        dl = None if draft_len is None else to_dev(np.ascontiguousarray(draft_len, np.int32))
        rt = None if row_temperature is None else to_dev(np.ascontiguousarray(row_temperature, np.float32))
        dsi = None if draft_stats_in is None else to_dev(np.ascontiguousarray(draft_stats_in, np.float64))
        tsi = None if target_stats_in is None else to_dev(np.ascontiguousarray(target_stats_in, np.float64))
        tstats = torch.full((B, g + 1, 2), float("nan"), dtype=torch.float64, device=DEV) if want_target_stats else None
        hb.hola_verify_ex(target_logits=P, draft_logits=D, draft_tokens=tok, seed=seed, B=B, gamma=g, V=V,
                          temperature=temperature, entropy_threshold=tau, out_accept_len=acc, out_next_token=nxt,
                          out_entropy=ent, workspace=ws, draft_len=dl, row_temperature=rt, draft_stats_in=dsi,
                          target_stats_out=tstats, target_stats_in=tsi, level=level, seq_base=seq_base)
    torch.cuda.synchronize()
    return GpuOut(acc.cpu().numpy(), nxt.cpu().numpy(), ent.cpu().numpy(),
                  None if tstats is None else tstats.cpu().numpy())


@dataclass
class Report:
    n_seq: int = 0
    accept_mismatch: int = 0          # tolerated (listed) accept-length differences
    token_mismatch: int = 0           # tolerated (listed) token differences
    listed_gate: int = 0              # oracle decisions with margin < 1e-6
    listed_ratio: int = 0
    listed_sample: int = 0
    max_entropy_abs: float = 0.0
    max_entropy_rel: float = 0.0

    def __str__(self):
        return (f"seq={self.n_seq} listed(gate/ratio/sample)={self.listed_gate}/{self.listed_ratio}/"
                f"{self.listed_sample} tolerated(accept/token)={self.accept_mismatch}/{self.token_mismatch} "
                f"entropy max abs={self.max_entropy_abs:.2e} rel={self.max_entropy_rel:.2e}")


def compare_level(target, draft, tokens, seed, temperature, tau, gpu: GpuOut, *, draft_len=None,
                  row_temperature=None, seq_base=0, level=0, entropy_rtol=None, num_threads=0) -> Report:
    """Run the oracle on the same (numpy) inputs and hold the GPU result to the parity bar."""
    call = orc.VerifyCall(target, draft, tokens, seed, temperature, tau, draft_len=draft_len,
                          row_temperature=row_temperature, level=level, seq_base=seq_base, num_threads=num_threads)
    ref = call.run()
    B, g = call.B, call.g
    lens = np.full(B, g, np.int32) if draft_len is None else np.asarray(draft_len, np.int32)
    if entropy_rtol is None:
        entropy_rtol = 1e-5 if np.asarray(target).dtype == np.float32 else 2e-3
    rep = Report(n_seq=B)

    # entropies (fp32 outputs on both sides; compare with the oracle's double)
    for b in range(B):
        L = int(lens[b])
        assert np.all(gpu.entropy[b, L:] == -1.0), f"seq {b}: entropy beyond draft_len must be -1"
        for j in range(L):
            h, hg = ref.entropy64[b, j], float(gpu.entropy[b, j])
            if np.isnan(h):
                assert np.isnan(hg), f"seq {b} pos {j}: oracle NaN entropy, gpu {hg}"
                continue
            err = abs(hg - h)
            rep.max_entropy_abs = max(rep.max_entropy_abs, err)
            rel = err / max(abs(h), 1e-30)
            if err > ENTROPY_ABS_FLOOR:
                rep.max_entropy_rel = max(rep.max_entropy_rel, rel)
                assert rel <= entropy_rtol, f"seq {b} pos {j}: entropy {hg} vs {h} rel {rel:.3e}"

    gm = np.where(np.isnan(ref.gate_margin), np.inf, ref.gate_margin)
    rm = np.where(np.isnan(ref.ratio_margin), np.inf, ref.ratio_margin)
    rep.listed_gate = int((gm < MARGIN).sum())
    rep.listed_ratio = int((rm < MARGIN).sum())
    rep.listed_sample = int((np.nan_to_num(ref.sample_margin, nan=np.inf) < MARGIN).sum())

    # accept lengths
    force = np.full(B, -1, np.int32)
    for b in range(B):
        ag, ao = int(gpu.accept_len[b]), int(ref.accept_len[b])
        assert 0 <= ag <= lens[b], f"seq {b}: accept_len {ag} outside [0, {lens[b]}]"
        if ag != ao:
            j = min(ag, ao)                               # the decision that differs
            assert min(gm[b, j], rm[b, j]) < MARGIN, (
                f"seq {b}: accept_len gpu {ag} vs oracle {ao}; deciding position {j} has margins "
                f"gate {gm[b, j]:.3e} ratio {rm[b, j]:.3e} (not listed near-threshold)")
            rep.accept_mismatch += 1
            force[b] = ag
    ref_tok, ref_smargin = ref.next_token.copy(), ref.sample_margin.copy()
    if (force >= 0).any():
        # judge the token of a flipped sequence against the oracle forced to the GPU's stop row
        call2 = orc.VerifyCall(target, draft, tokens, seed, temperature, tau, draft_len=draft_len,
                               row_temperature=row_temperature, level=level, seq_base=seq_base,
                               force_accept_len=force, num_threads=num_threads)
        ref2 = call2.run()
        sel = force >= 0
        ref_tok[sel], ref_smargin[sel] = ref2.next_token[sel], ref2.sample_margin[sel]

    # next tokens
    for b in range(B):
        tg, to = int(gpu.next_token[b]), int(ref_tok[b])
        if tg == to:
            continue
        assert ref_smargin[b] < MARGIN, (
            f"seq {b}: next_token gpu {tg} vs oracle {to}, sample margin {ref_smargin[b]:.3e} (not listed)")
        iv = call.sample_interval(b, int(gpu.accept_len[b]), tg)
        assert iv is not None, f"seq {b}: gpu token {tg} has no interval"
        u2 = orc.hsd_uniforms(seed, seq_base + b, int(gpu.accept_len[b]), level)[1]
        assert iv[0] - MARGIN <= u2 <= iv[1] + MARGIN and iv[1] > iv[0], (
            f"seq {b}: gpu token {tg} interval {iv} does not hold u'={u2}")
        rep.token_mismatch += 1
    return rep
