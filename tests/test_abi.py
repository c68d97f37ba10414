"""The C-ABI library loads without a GPU, exports every symbol include/hola.h declares, and its host
logic (argument checks, workspace sizing, status strings) behaves as the header states.  No compute."""
import ctypes as C
import os
import re

import pytest

from conftest import ROOT
from paper_2506_18952_amd import binding as hb


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "hola.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hola_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    names = _declared_functions()
    assert len(names) >= 16
    L = hb.lib()
    for n in names:
        assert hasattr(L, n), f"{n} declared in include/hola.h but not exported"
    assert set(names) == set(hb.EXPORTS)


def test_status_strings_and_version():
    L = hb.lib()
    seen = {L.hola_status_string(i) for i in range(5)}
    assert len(seen) == 5 and all(seen)
    assert b"gfx950" in L.hola_version()


def test_workspace_bytes():
    assert hb.hola_workspace_bytes(0, 4, 100) > 0
    assert hb.hola_workspace_bytes(4, 0, 100) == 0           # gamma < 1
    assert hb.hola_workspace_bytes(4, 64, 100) == 0          # gamma > 63
    assert hb.hola_workspace_bytes(4, 63, 100) > 0
    assert hb.hola_workspace_bytes(4, 4, 0) == 0
    assert hb.hola_workspace_bytes(-1, 4, 100) == 0
    a, b, c = (hb.hola_workspace_bytes(*s) for s in ((8, 4, 1000), (16, 4, 1000), (16, 8, 128256)))
    assert a < b < c
    # the headline shape: ~9 MB of partial sums plus 16 KB of candidate list per row for filtered calls
    assert hb.hola_workspace_bytes(256, 8, 128256) < 96 << 20
    # the candidate lists are left out (and the per-row filter kernel used) before they pass 256 MB
    assert hb.hola_workspace_bytes(8192, 8, 128256) < hb.hola_workspace_bytes(256, 8, 128256) * 32
    assert hb.hola_hsd_workspace_bytes(3, 128, 8, 151936) > hb.hola_workspace_bytes(128, 9, 151936)
    assert hb.hola_hsd_workspace_bytes(1, 8, 4, 100) == 0    # needs at least two models
    assert hb.hola_hsd_workspace_bytes(3, 8, 63, 100) == 0   # gamma grows past the limit


def test_workspace_bytes_of_one_call():
    """A call without filters does not pay for the filters' candidate lists."""
    full = hb.hola_workspace_bytes(256, 8, 128256)
    plain = hb.hola_workspace_bytes_ex(256, 8, 128256)
    assert 0 < plain < 12 << 20 < full                       # ~9 MB of partial sums against ~82 MB
    assert hb.hola_workspace_bytes_ex(256, 8, 128256, top_k=50) == full
    assert hb.hola_workspace_bytes_ex(256, 8, 128256, top_p=0.9) == full
    assert hb.hola_workspace_bytes_ex(256, 8, 128256, top_k=128256, top_p=1.0) == plain   # both filters off
    assert hb.hola_workspace_bytes_ex(4, 0, 100) == 0 and hb.lib().hola_workspace_bytes_ex(None) == 0
    a = _args(workspace_bytes=hb.hola_workspace_bytes_ex(4, 3, 100))
    a.B = 0
    assert hb.lib().hola_verify_ex(C.byref(a)) == hb.HOLA_OK
    a = _args(workspace_bytes=hb.hola_workspace_bytes_ex(4, 3, 100) - 1)
    assert hb.lib().hola_verify_ex(C.byref(a)) == hb.HOLA_ERR_WORKSPACE
    a = _args(workspace_bytes=hb.hola_workspace_bytes_ex(4, 3, 100), top_k=5)      # a filtered call needs the larger one
    assert hb.lib().hola_verify_ex(C.byref(a)) == hb.HOLA_ERR_WORKSPACE


def test_tuning_of_one_call_is_validated():
    for bad in (dict(stats_split=99), dict(stats_unroll=3), dict(path=7), dict(fused_waves=5), dict(filter_path=2),
                dict(tail_split=3), dict(tail_split=16)):
        t = hb.Tuning(**bad)
        a = _args(tuning=C.pointer(t))
        assert hb.lib().hola_verify_ex(C.byref(a)) == hb.HOLA_ERR_INVALID_ARG
        ta = _tree_args(tuning=C.pointer(t))
        assert hb.lib().hola_verify_tree(C.byref(ta)) == hb.HOLA_ERR_INVALID_ARG


def test_thread_defaults_do_not_leak_between_threads():
    """hola_set_tuning acts on the calling thread alone: an invalid value is refused where it is set, and a second
    thread starts from the built-in defaults whatever the first one chose."""
    import threading
    hb.hola_set_tuning(stats_split=4, path=hb.PATH_SPLIT4)
    seen = {}

    def other():
        seen["status"] = hb.lib().hola_set_tuning(None)          # restoring defaults in this thread only
    th = threading.Thread(target=other)
    th.start(); th.join()
    assert seen["status"] == hb.HOLA_OK
    hb.hola_set_tuning()


def _args(**kw):
    a = hb.VerifyArgs()
    fake = 0x1000                                             # never dereferenced: checks come first
    a.target_logits = a.draft_logits = a.draft_tokens = fake
    a.out_accept_len = a.out_next_token = fake
    a.dtype, a.B, a.gamma, a.V = hb.HOLA_DTYPE_BF16, 4, 3, 100
    a.temperature, a.entropy_threshold = 1.0, 2.0
    a.workspace, a.workspace_bytes = 0x10000, 1 << 30
    for k, v in kw.items():
        setattr(a, k, v)
    return a


@pytest.mark.parametrize("kw,want", [
    (dict(B=-1), hb.HOLA_ERR_INVALID_ARG),
    (dict(gamma=0), hb.HOLA_ERR_INVALID_ARG),
    (dict(gamma=64), hb.HOLA_ERR_INVALID_ARG),
    (dict(V=0), hb.HOLA_ERR_INVALID_ARG),
    (dict(dtype=7), hb.HOLA_ERR_UNSUPPORTED),
    (dict(target_logits=None), hb.HOLA_ERR_INVALID_ARG),
    (dict(draft_logits=None), hb.HOLA_ERR_INVALID_ARG),
    (dict(draft_tokens=None), hb.HOLA_ERR_INVALID_ARG),
    (dict(out_accept_len=None), hb.HOLA_ERR_INVALID_ARG),
    (dict(out_next_token=None), hb.HOLA_ERR_INVALID_ARG),
    (dict(target_logits=0x1001), hb.HOLA_ERR_INVALID_ARG),    # not aligned to the element size
    (dict(target_ld=99), hb.HOLA_ERR_INVALID_ARG),
    (dict(draft_ld=50), hb.HOLA_ERR_INVALID_ARG),
    (dict(entropy_ld=2), hb.HOLA_ERR_INVALID_ARG),
    (dict(temperature=-0.5), hb.HOLA_ERR_INVALID_ARG),
    (dict(temperature=float("nan")), hb.HOLA_ERR_INVALID_ARG),
    (dict(temperature=float("inf")), hb.HOLA_ERR_INVALID_ARG),
    (dict(entropy_threshold=float("nan")), hb.HOLA_ERR_INVALID_ARG),
    (dict(workspace=None), hb.HOLA_ERR_WORKSPACE),
    (dict(workspace=0x10010), hb.HOLA_ERR_WORKSPACE),         # not 256-byte aligned
    (dict(workspace_bytes=1024), hb.HOLA_ERR_WORKSPACE),
    (dict(B=0), hb.HOLA_OK),                                  # empty batch: successful no-op
])
def test_verify_ex_argument_errors(kw, want):
    a = _args(**kw)
    assert hb.lib().hola_verify_ex(C.byref(a)) == want


def _tree_args(**kw):
    a = hb.TreeArgs()
    fake = 0x1000
    a.target_logits = a.draft_logits = a.node_token = a.node_parent = fake
    a.out_accept_len = a.out_next_token = fake
    a.dtype, a.B, a.N, a.V = hb.HOLA_DTYPE_BF16, 4, 6, 100
    a.temperature, a.entropy_threshold = 1.0, 2.0
    a.workspace, a.workspace_bytes = 0x10000, 1 << 30
    for k, v in kw.items():
        setattr(a, k, v)
    return a


@pytest.mark.parametrize("kw,want", [
    (dict(B=-1), hb.HOLA_ERR_INVALID_ARG),
    (dict(N=0), hb.HOLA_ERR_INVALID_ARG),
    (dict(N=64), hb.HOLA_ERR_INVALID_ARG),
    (dict(V=0), hb.HOLA_ERR_INVALID_ARG),
    (dict(dtype=3), hb.HOLA_ERR_UNSUPPORTED),
    (dict(target_logits=None), hb.HOLA_ERR_INVALID_ARG),
    (dict(draft_logits=None), hb.HOLA_ERR_INVALID_ARG),
    (dict(node_token=None), hb.HOLA_ERR_INVALID_ARG),
    (dict(node_parent=None), hb.HOLA_ERR_INVALID_ARG),
    (dict(out_accept_len=None), hb.HOLA_ERR_INVALID_ARG),
    (dict(out_next_token=None), hb.HOLA_ERR_INVALID_ARG),
    (dict(draft_logits=0x1001), hb.HOLA_ERR_INVALID_ARG),
    (dict(target_ld=99), hb.HOLA_ERR_INVALID_ARG),
    (dict(temperature=float("nan")), hb.HOLA_ERR_INVALID_ARG),
    (dict(temperature=-1.0), hb.HOLA_ERR_INVALID_ARG),
    (dict(temperature=0.0), hb.HOLA_ERR_UNSUPPORTED),         # greedy rows are not taken on trees
    (dict(entropy_threshold=float("nan")), hb.HOLA_ERR_INVALID_ARG),
    (dict(V=1 << 23, dtype=hb.HOLA_DTYPE_F32), hb.HOLA_ERR_UNSUPPORTED),   # more sampler tiles than the tail kernel holds
    (dict(workspace=None), hb.HOLA_ERR_WORKSPACE),
    (dict(workspace=0x10040), hb.HOLA_ERR_WORKSPACE),
    (dict(workspace_bytes=4096), hb.HOLA_ERR_WORKSPACE),
    (dict(B=0), hb.HOLA_OK),
])
def test_verify_tree_argument_errors(kw, want):
    a = _tree_args(**kw)
    assert hb.lib().hola_verify_tree(C.byref(a)) == want
    assert hb.lib().hola_verify_tree(None) == hb.HOLA_ERR_INVALID_ARG


def test_tree_workspace_bytes():
    assert hb.hola_tree_workspace_bytes(4, 0, 100) == 0 and hb.hola_tree_workspace_bytes(4, 64, 100) == 0
    assert 0 < hb.hola_tree_workspace_bytes(4, 63, 100) <= hb.hola_workspace_bytes(4, 63, 100)
    assert hb.hola_tree_workspace_bytes(256, 16, 128256) < 20 << 20      # the row partials alone


def test_null_args_and_short_forms():
    L = hb.lib()
    assert L.hola_verify_ex(None) == hb.HOLA_ERR_INVALID_ARG
    f = 0x1000
    for fn in (L.hola_verify_f32, L.hola_verify_bf16):
        assert fn(None, f, f, 0, 2, 2, 10, 1.0, 1.0, f, f, f, None) == hb.HOLA_ERR_INVALID_ARG
        assert fn(f, f, f, 0, 2, 0, 10, 1.0, 1.0, f, f, f, None) == hb.HOLA_ERR_INVALID_ARG
        assert fn(f, f, f, 0, 2, 2, 10, 0.0, 1.0, f, f, f, None) == hb.HOLA_ERR_INVALID_ARG   # no greedy short form
        assert fn(f, f, f, 0, 0, 2, 10, 1.0, 1.0, f, f, f, None) == hb.HOLA_OK
    assert L.hola_row_stats(None, 0, 0, 4, 10, 1.0, f, 0x10000, 1 << 30, None) == hb.HOLA_ERR_INVALID_ARG
    assert L.hola_row_stats(f, 0, 0, 4, 10, 0.0, f, 0x10000, 1 << 30, None) == hb.HOLA_ERR_INVALID_ARG
    assert L.hola_row_stats(f, 0, 0, 0, 10, 1.0, f, 0x10000, 1 << 30, None) == hb.HOLA_OK
    taus = (C.c_float * 2)(1.0, 2.0)
    models = (hb.ModelLogits * 3)()
    assert L.hola_hsd_verify(models, 3, 1, f, 0, 0, 4, 2, 10, None, 1.0, taus, f, f, f, None, 0x10000, 1 << 30,
                             None) == hb.HOLA_ERR_INVALID_ARG                                 # NULL model logits
    for m in models:
        m.logits = f
    assert L.hola_hsd_verify(models, 3, 1, f, 0, 0, 4, 2, 10, None, 1.0, taus, f, f, f, None, 0x10000, 16,
                             None) == hb.HOLA_ERR_WORKSPACE
    assert L.hola_hsd_verify(models, 1, 1, f, 0, 0, 4, 2, 10, None, 1.0, taus, f, f, f, None, 0x10000, 1 << 30,
                             None) == hb.HOLA_ERR_INVALID_ARG


def test_tuning_validation():
    hb.hola_set_tuning(2, 4, 0)
    with pytest.raises(hb.HolaError):
        hb.hola_set_tuning(0, 3, 0)
    with pytest.raises(hb.HolaError):
        hb.hola_set_tuning(99, 0, 0)
    hb.hola_set_tuning()


def test_product_does_not_import_the_oracle():
    """The HIP path's Python and C++ sources never name the oracle."""
    pkg = os.path.join(ROOT, "paper_2506_18952_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "hola_oracle" not in text and "from oracle" not in text and "import oracle" not in text, f


def test_tile_entry_points_argument_checks():
    L = hb.lib()
    f = 0x1000
    assert hb.hola_tile_stats_workspace_bytes(4, 1000, 128) > 0
    assert hb.hola_tile_stats_workspace_bytes(4, 1000, 0) == 0
    assert hb.hola_tile_stats_workspace_bytes(-1, 1000, 128) == 0
    assert hb.hola_tile_stats_workspace_bytes(8, 1000, 10) > hb.hola_tile_stats_workspace_bytes(8, 1000, 500)
    ws, wb = 0x10000, 1 << 30
    assert L.hola_tile_stats(f, 0, 0, 4, 100, 0, 1.0, f, ws, wb, None) == hb.HOLA_ERR_INVALID_ARG      # tile_cols < 1
    assert L.hola_tile_stats(None, 0, 0, 4, 100, 10, 1.0, f, ws, wb, None) == hb.HOLA_ERR_INVALID_ARG
    assert L.hola_tile_stats(f, 0, 0, 4, 100, 10, 0.0, f, ws, wb, None) == hb.HOLA_ERR_INVALID_ARG     # T must be > 0
    assert L.hola_tile_stats(f, 0, 50, 4, 100, 10, 1.0, f, ws, wb, None) == hb.HOLA_ERR_INVALID_ARG    # ld < V
    assert L.hola_tile_stats(f, 5, 0, 4, 100, 10, 1.0, f, ws, wb, None) == hb.HOLA_ERR_UNSUPPORTED
    assert L.hola_tile_stats(f, 0, 0, 4, 100, 10, 1.0, f, ws, 64, None) == hb.HOLA_ERR_WORKSPACE
    assert L.hola_tile_stats(f, 0, 0, 0, 100, 10, 1.0, f, ws, wb, None) == hb.HOLA_OK                  # no rows
    assert L.hola_merge_tile_stats(None, 4, 3, f, None) == hb.HOLA_ERR_INVALID_ARG
    assert L.hola_merge_tile_stats(f, 4, 0, f, None) == hb.HOLA_ERR_INVALID_ARG
    assert L.hola_merge_tile_stats(f, 0, 3, f, None) == hb.HOLA_OK


def test_supplied_target_statistics_argument_checks():
    a = _args(target_stats_in=0x2000)
    a.row_temperature = 0x3000
    assert hb.lib().hola_verify_ex(C.byref(a)) == hb.HOLA_ERR_UNSUPPORTED
    a = _args(target_stats_in=0x2000, temperature=0.0)
    assert hb.lib().hola_verify_ex(C.byref(a)) == hb.HOLA_ERR_UNSUPPORTED


def test_header_is_plain_c_and_matches_the_binding(tmp_path):
    """include/hola.h compiles as C99 without warnings, and every structure of the binding has the size and the
    field offsets the C compiler gives the header's (same field names, same order)."""
    import ctypes as C
    import re
    import shutil
    import subprocess

    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    pairs = [("hola_verify_args", hb.VerifyArgs), ("hola_model_logits", hb.ModelLogits), ("hola_hsd_args", hb.HsdArgs), ("hola_tree_args", hb.TreeArgs),
             ("hola_tuning", hb.Tuning)]
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "hola.h"', 'int main(void) {']
    for cname, cls in pairs:
        lines.append(f'  printf("{cname} size %zu\\n", sizeof({cname}));')
        for fname, _ in cls._fields_:
            lines.append(f'  printf("{cname} {fname} %zu\\n", offsetof({cname}, {fname}));')
    lines += ['  return 0;', '}']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(root, "include"),
                    str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout
    got = {}
    for m in re.finditer(r"(\w+) (\w+) (\d+)", out):
        got[(m.group(1), m.group(2))] = int(m.group(3))
    for cname, cls in pairs:
        assert got[(cname, "size")] == C.sizeof(cls), cname
        for fname, _ in cls._fields_:
            assert got[(cname, fname)] == getattr(cls, fname).offset, (cname, fname)
