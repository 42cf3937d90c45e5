"""Host-side checks of the C ABI (no GPU needed): the library loads, exports every
symbol the header declares, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

import paper_2310_18547_amd as sg


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "sgmv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sgmv_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    names = _declared_functions()
    assert {"sgmv_shrink", "sgmv_expand", "sgmv_add_lora", "sgmv_workspace_bytes",
            "sgmv_validate_segments", "sgmv_status_string"} <= set(names)
    L = ctypes.CDLL(sg.library_path())
    for n in names:
        assert hasattr(L, n), n


def test_struct_layout_matches_header():
    # 10 int32 fields, pointer, size_t
    assert ctypes.sizeof(sg.SgmvProblem) == 12 * 4 + 8 + 8
    assert sg.SgmvProblem.workspace.offset == 48


def test_status_strings():
    seen = {sg.sgmv_status_string(i) for i in range(9)}
    assert len(seen) == 9 and "unknown status" not in seen
    assert sg.sgmv_status_string(99) == "unknown status"


def test_workspace_bytes():
    assert sg.sgmv_workspace_bytes(0, 16) == 0
    assert sg.sgmv_workspace_bytes(-3, 16) == 0
    for T in (1, 7, 64, 1000, 4608, 100000):
        for r in (8, 16, 32, 64):
            b = sg.sgmv_workspace_bytes(T, r)
            assert b >= 1024 + 3 * 16 * T * r * 4 + T * r * 4 + T * 4   # header, >= 16 slices, exchange, operands
            assert b <= 1024 + 3 * (64 * T * r * 4 + 256) + T * r * 4 + T * 4 + 768 and b % 256 == 0
    assert sg.sgmv_workspace_bytes(64, 16) == 1024 + 3 * 64 * 64 * 16 * 4 + 2 * 2048 + 256


def test_validate_segments():
    ok = np.array([0, 1, 4, 4, 8], np.int32)
    assert sg.sgmv_validate_segments(ok, 4, 8) == 0
    assert sg.sgmv_validate_segments(ok, 4, 9) == 2
    assert sg.sgmv_validate_segments(np.array([1, 2], np.int32), 1, 2) == 2
    assert sg.sgmv_validate_segments(np.array([0, 3, 2], np.int32), 2, 2) == 2
    assert sg.sgmv_validate_segments(None, 1, 1) == 1
    assert sg.sgmv_validate_segments(ok, -1, 8) == 2
    assert sg.sgmv_validate_segments(np.array([0], np.int32), 0, 0) == 0


FAKE = 0x10000   # a non-null, aligned address that is never dereferenced on these paths


def _prob(**kw):
    d = dict(dtype=sg.F16, h_in=4096, h_out=4096, r=16, num_layers=4, n_tokens=8,
             workspace=FAKE, workspace_bytes=1 << 30)
    d.update(kw)
    return sg.make_problem(**d)


def _add(p, y=FAKE, x=FAKE, A=FAKE, B=FAKE, s=FAKE, n=2, layer=0):
    return sg.sgmv_add_lora(p, y, x, A, B, s, n, layer, 1.0, check=False)


def test_argument_errors_are_reported_without_a_device():
    assert _add(_prob(dtype=7)) == 3
    assert _add(_prob(r=12)) == 3
    assert _add(_prob(r=128)) == 3
    assert _add(_prob(h_in=4100)) == 3
    assert _add(_prob(h_out=12)) == 3
    assert _add(_prob(h_in=0)) == 2
    assert _add(_prob(n_tokens=-1)) == 2
    assert _add(_prob(num_layers=0)) == 2
    assert _add(_prob(), n=-1) == 2
    assert _add(_prob(), layer=4) == 6
    assert _add(_prob(), layer=-1) == 6
    assert _add(_prob(), y=None) == 1
    assert _add(_prob(), x=None) == 1
    assert _add(_prob(), A=None) == 1
    assert _add(_prob(), B=None) == 1
    assert _add(_prob(), s=None) == 1
    assert _add(_prob(), x=FAKE + 2) == 4
    assert _add(_prob(), y=FAKE + 8) == 4
    assert _add(_prob(workspace=None)) == 5
    assert _add(_prob(workspace=FAKE + 16)) == 4
    assert _add(_prob(workspace_bytes=16)) == 5
    assert _add(_prob(path=9)) == 3
    assert _add(_prob(path=sg.PATH_FUSED)) == 3            # workspace not declared ready
    assert _add(_prob(path=sg.PATH_FUSED, workspace_ready=1, max_seg_len=0)) == 3
    assert _add(_prob(path=sg.PATH_FUSED, workspace_ready=1, max_seg_len=65)) == 3
    assert sg.sgmv_workspace_init(None, 1024, check=False) == 1
    assert sg.sgmv_workspace_init(FAKE + 8, 1024, check=False) == 4
    assert sg.sgmv_workspace_check(None) == 1
    assert sg.sgmv_workspace_init(FAKE, 16, check=False) == 5
    assert _add(_prob(ksplit=1000)) == 3
    assert _add(_prob(expand_threads=100)) == 3
    # nothing to do: OK without any launch
    assert _add(_prob(), n=0) == 0
    assert _add(_prob(n_tokens=0)) == 0
    with pytest.raises(sg.SgmvError):
        sg.sgmv_add_lora(_prob(r=12), FAKE, FAKE, FAKE, FAKE, FAKE, 2, 0, 1.0)


def test_shrink_and_expand_argument_errors():
    p = _prob()
    assert sg.sgmv_shrink(p, None, FAKE, FAKE, FAKE, 2, 0, check=False) == 1
    assert sg.sgmv_shrink(p, FAKE + 4, FAKE, FAKE, FAKE, 2, 0, check=False) == 4
    assert sg.sgmv_shrink(_prob(workspace=None), FAKE, FAKE, FAKE, FAKE, 2, 0, check=False) == 5
    assert sg.sgmv_shrink(_prob(h_out=0), FAKE, FAKE, FAKE, FAKE, 0, 0, check=False) == 0   # h_out ignored
    assert sg.sgmv_expand(p, FAKE, None, FAKE, FAKE, 2, 0, 1.0, check=False) == 1
    assert sg.sgmv_expand(_prob(workspace=None, h_in=0), FAKE, FAKE, FAKE, FAKE, 0, 0, 1.0,
                          check=False) == 0                                               # no workspace, h_in ignored
    assert sg.sgmv_expand(p, FAKE, FAKE, FAKE, FAKE, 2, 9, 1.0, check=False) == 6


def test_accounting_against_paper_closed_forms():
    from paper_2310_18547_amd import accounting as acc
    path = os.path.join(ROOT, "tests", "golden", "roofline_closed_forms.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 6
    for s_n, n, h_i, h_o, flop, io in (map(int, r) for r in rows):
        assert acc.paper_flop(s_n, h_i, h_o) == flop
        assert acc.paper_io_bytes(s_n, n, h_i, h_o) == io
    # the finer count used for the roofline at the metric configuration
    assert acc.algorithmic_bytes("shrink", 64, 64, 4096, 4096, 16) == 8916992
    assert acc.algorithmic_bytes("expand", 64, 64, 4096, 4096, 16) == 9441280
    assert acc.algorithmic_bytes("add_lora", 64, 64, 4096, 4096, 16) == 18358272
    assert acc.algorithmic_bytes("add_lora", 1, 1, 4096, 4096, 16) == 286848
    assert acc.flops("add_lora", 64, 4096, 4096, 16) == 16777216
    # it differs from the paper's form only by counting y twice and v as fp32
    paper = acc.paper_io_bytes(64, 64, 4096, 16) + acc.paper_io_bytes(64, 64, 16, 4096)
    assert acc.algorithmic_bytes("add_lora", 64, 64, 4096, 4096, 16) - paper == 64 * 4096 * 2 + 2 * 64 * 16 * 2
