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
    seen = {sg.sgmv_status_string(i) for i in range(10)}
    assert len(seen) == 10 and "unknown status" not in seen
    assert sg.sgmv_status_string(99) == "unknown status"


HEADER = 1024 * 4 + 256   # generation copies (1024 x 32 bit), error word and padding


def test_workspace_bytes():
    assert sg.sgmv_workspace_bytes(0, 16) == 0
    assert sg.sgmv_workspace_bytes(-3, 16) == 0
    for T in (1, 7, 64, 1000, 4608, 100000):
        for r in (8, 16, 32, 64):
            b = sg.sgmv_workspace_bytes(T, r)
            assert b >= HEADER + 3 * 16 * T * r * 4 + T * r * 4 + T * 4   # header, >= 16 slices, exchange, operands
            assert b <= HEADER + 3 * (64 * T * r * 4 + 256) + T * r * 4 + T * 4 + 768 and b % 256 == 0
    assert sg.sgmv_workspace_bytes(64, 16) == HEADER + 3 * 64 * 64 * 16 * 4 + 2 * 2048 + 256


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
    assert _add(_prob(path=sg.PATH_MATRIX, n_tokens=70000), n=70000) == 3   # more segments than the MFMA grid takes
    assert _add(_prob(path=sg.PATH_FUSED)) == 3            # workspace not declared ready
    assert _add(_prob(path=sg.PATH_FUSED, workspace_ready=1, max_seg_len=0)) == 3
    assert _add(_prob(path=sg.PATH_FUSED, workspace_ready=1, max_seg_len=5000)) == 3
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


def _plan(n_segs, n_proj=1, **kw):
    kw.setdefault("workspace_ready", 1)
    p = _prob(**kw)
    rc, plan = sg.sgmv_plan_add_lora(p, n_segs, n_proj, check=False)
    return rc, plan


def test_plan_single_launch_shapes():
    """Launch policy of sgmv_add_lora, asked of the library (host-only, no device)."""
    # one row per segment: the row kernel with the hand-off, S a power of two with S * segments <=
    # 256 units; its grid is padded to whole rows of eight segments (a segment's workgroups share an XCD).
    # Beyond 128 rows of 4096 features, which would need two slices each and two workgroups per unit,
    # the single-launch kernel without hand-off takes over up to several hundred segments, then the
    # launch-per-step kernels; a forced path still takes what was asked for
    rc, pl = _plan(256, n_tokens=256, max_seg_len=1)
    assert rc == 0 and pl.kernel == sg.KERNEL_WHOLE and (pl.launches, pl.slices, pl.workgroups) == (1, 1, 256)
    rc, pl = _plan(1024, n_tokens=1024, max_seg_len=1)
    assert rc == 0 and pl.kernel == sg.KERNEL_VECTOR
    rc, pl = _plan(256, n_tokens=256, max_seg_len=1, path=sg.PATH_FUSED)
    assert rc == 0 and pl.kernel == sg.KERNEL_FUSED and (pl.slices, pl.workgroups) == (2, 512)
    rc, pl = _plan(256, n_tokens=256, max_seg_len=1, h_in=2048)       # A_i of 64 KB: no hand-off
    assert rc == 0 and pl.kernel == sg.KERNEL_WHOLE and (pl.slices, pl.workgroups) == (1, 256)
    rc, pl = _plan(256, n_tokens=256, max_seg_len=1, h_in=2048, path=sg.PATH_FUSED)
    assert rc == 0 and pl.kernel == sg.KERNEL_FUSED and (pl.slices, pl.workgroups) == (1, 256)
    rc, pl = _plan(4, n_tokens=8, max_seg_len=3, h_in=256, h_out=256, r=8)   # longer segments, small A_i: the same per row
    assert rc == 0 and pl.kernel == sg.KERNEL_WHOLE and pl.workgroups == 8 * pl.slices
    rc, pl = _plan(8, n_tokens=8, max_seg_len=1, h_in=1024, h_out=1024)    # narrow: one slice ...
    assert rc == 0 and pl.kernel == sg.KERNEL_WHOLE
    rc, pl = _plan(8, n_tokens=8, max_seg_len=1, h_in=1024, h_out=1024, path=sg.PATH_FUSED)
    assert rc == 0 and pl.kernel == sg.KERNEL_FUSED and pl.slices == 1
    rc, pl = _plan(8, n_tokens=8, max_seg_len=1, h_in=2048, h_out=2048, r=64, path=sg.PATH_FUSED)   # ... or what leaves a slice a full batch of loads
    assert rc == 0 and pl.kernel == sg.KERNEL_FUSED and pl.slices == 8
    for batch, S in ((1, 8), (8, 8), (16, 8), (32, 8), (48, 4), (64, 4), (96, 2), (128, 4)):
        rc, pl = _plan(batch, n_tokens=batch, max_seg_len=1)
        assert rc == 0 and pl.kernel == sg.KERNEL_FUSED and pl.launches == 1
        assert (pl.slices, pl.workgroups) == (S, S * batch), (batch, pl.slices)
    rc, pl = _plan(12, n_tokens=12, max_seg_len=1)
    assert rc == 0 and pl.kernel == sg.KERNEL_FUSED and (pl.slices, pl.workgroups) == (8, 8 * 16)   # two rows of eight
    # rank 8 (small A_i): every workgroup computes the whole shrink itself, no hand-off
    for batch, S in ((1, 8), (16, 8), (64, 4), (256, 1)):
        rc, pl = _plan(batch, n_tokens=batch, max_seg_len=1, r=8)
        assert rc == 0 and pl.kernel == sg.KERNEL_WHOLE and (pl.launches, pl.slices) == (1, S)
        assert pl.workgroups == 8 * S * ((batch + 7) // 8)
    # binary16 rows so wide that the hand-off kernel needs an odd number of slices: the kernel without
    # hand-off once those slices outnumber the compute units
    for batch, kernel in ((80, sg.KERNEL_FUSED), (96, sg.KERNEL_WHOLE), (128, sg.KERNEL_WHOLE)):
        rc, pl = _plan(batch, n_tokens=batch, max_seg_len=1, h_in=5120, h_out=5120)
        assert rc == 0 and pl.kernel == kernel, (batch, pl.kernel)
    rc, pl = _plan(128, n_tokens=128, max_seg_len=1, h_in=5120, h_out=5120, dtype=sg.BF16)
    assert rc == 0 and pl.kernel == sg.KERNEL_FUSED and pl.slices == 3
    # rank 8 with a large A_i: the hand-off kernel again (the whole-shrink kernel re-reads A_i per slice)
    for h, batch, kernel in ((4096, 64, sg.KERNEL_WHOLE), (5120, 32, sg.KERNEL_FUSED), (5120, 64, sg.KERNEL_FUSED),
                             (8192, 1, sg.KERNEL_FUSED), (8192, 64, sg.KERNEL_FUSED)):
        rc, pl = _plan(batch, n_tokens=batch, max_seg_len=1, r=8, h_in=h, h_out=h)
        assert rc == 0 and pl.kernel == kernel, (h, batch, pl.kernel)
    # from rank 32 on no single launch whose workgroups would fill the units unevenly (288, 384 of 256)
    rc, pl = _plan(96, n_tokens=96, max_seg_len=1, r=32, h_in=5120, h_out=5120)
    assert rc == 0 and pl.kernel == sg.KERNEL_VECTOR
    rc, pl = _plan(96, n_tokens=96, max_seg_len=1, r=64, h_in=8192, h_out=8192)
    assert rc == 0 and pl.kernel == sg.KERNEL_VECTOR
    rc, pl = _plan(128, n_tokens=128, max_seg_len=1, r=32)
    assert rc == 0 and pl.kernel == sg.KERNEL_FUSED and pl.workgroups == 512
    # sixteen slices for small batches from rank 32 on, by the wider of input and output
    rc, pl = _plan(8, n_tokens=8, max_seg_len=1, r=32, h_in=4096, h_out=11008)
    assert rc == 0 and pl.kernel == sg.KERNEL_FUSED and pl.slices == 16
    rc, pl = _plan(8, n_tokens=8, max_seg_len=1, r=16, h_in=11008, h_out=4096)
    assert rc == 0 and pl.kernel == sg.KERNEL_FUSED and pl.slices == 8
    # that kernel needs no workspace: it is what a caller without a prepared one gets, and forced
    # it runs without any
    rc, pl = _plan(64, n_tokens=64, max_seg_len=1, workspace_ready=0)
    assert rc == 0 and pl.kernel == sg.KERNEL_WHOLE and pl.launches == 1
    rc, pl = _plan(64, n_tokens=64, max_seg_len=1, path=sg.PATH_WHOLE, workspace=None, workspace_bytes=0)
    assert rc == 0 and pl.kernel == sg.KERNEL_WHOLE
    rc, pl = _plan(64, n_tokens=64, max_seg_len=3, path=sg.PATH_WHOLE)
    assert rc == 3                                   # one-row segments only
    rc, pl = _plan(64, n_tokens=64, max_seg_len=1, path=sg.PATH_WHOLE, h_in=11008)
    assert rc == 3                                   # input rows wider than a workgroup stages
    # short multi-row segments in a small batch (or segments of unknown length): the one-row kernel
    # run per ROW of the batch, every row looking its segment up
    for kw in (dict(n_tokens=64, max_seg_len=5), dict(n_tokens=64, max_seg_len=0), dict(n_tokens=64, max_seg_len=64)):
        rc, pl = _plan(39, **kw)
        assert rc == 0 and pl.kernel == sg.KERNEL_FUSED and (pl.launches, pl.slices, pl.workgroups) == (1, 4, 256)
    rc, pl = _plan(64, n_tokens=200, max_seg_len=0)          # ranks up to 16: up to 256 rows where the tile kernel is out
    assert rc == 0 and pl.kernel == sg.KERNEL_FUSED and (pl.slices, pl.workgroups) == (2, 400)
    rc, pl = _plan(39, n_tokens=64, max_seg_len=5, path=sg.PATH_ROWS)
    assert rc == 0 and pl.kernel == sg.KERNEL_FUSED and pl.workgroups == 256
    # a batch of mostly empty segments (the look-up takes a round per 64 of them): not by itself
    rc, pl = _plan(300, n_tokens=64, max_seg_len=5)
    assert rc == 0 and pl.kernel != sg.KERNEL_FUSED
    rc, pl = _plan(300, n_tokens=64, max_seg_len=5, path=sg.PATH_ROWS)
    assert rc == 0 and pl.kernel == sg.KERNEL_FUSED
    rc, pl = _plan(39, n_tokens=2000, max_seg_len=60, path=sg.PATH_ROWS)
    assert rc == 3                                   # more rows than the launch takes workgroups
    # in larger batches (or when asked for): sixteen-row tiles, every workgroup resident
    for kw in (dict(n_tokens=64, max_seg_len=5, path=sg.PATH_FUSED), dict(n_tokens=300, max_seg_len=12)):
        rc, pl = _plan(39, **kw)
        assert rc == 0 and pl.kernel == sg.KERNEL_TILE and pl.launches == 1
        assert pl.slices * 39 <= 256 and pl.workgroups == pl.slices * 39
        assert 0 < pl.lds_bytes <= 160 * 1024
    rc, pl = _plan(1, n_tokens=64, max_seg_len=64, path=sg.PATH_FUSED)
    assert rc == 0 and pl.kernel == sg.KERNEL_TILE and pl.workgroups == pl.slices * 4
    # without the prepared workspace the kernels with a hand-off are not taken
    rc, pl = _plan(64, n_tokens=64, max_seg_len=1, workspace_ready=0, r=64)
    assert rc == 0 and pl.kernel == sg.KERNEL_VECTOR and pl.launches == 2
    rc, pl = _plan(39, n_tokens=64, max_seg_len=5, workspace_ready=0)
    assert rc == 0 and pl.kernel == sg.KERNEL_VECTOR   # many short segments: work by rows, not by 64-row blocks
    rc, pl = _plan(16, n_tokens=128, max_seg_len=8, workspace_ready=0)
    assert rc == 0 and pl.kernel == sg.KERNEL_MATRIX
    # rank 64: per row up to 64 rows; beyond, the tile kernel up to eight rows per segment, then the
    # MFMA kernels, which also take few short segments there
    rc, pl = _plan(8, n_tokens=64, max_seg_len=8, r=64)
    assert rc == 0 and pl.kernel == sg.KERNEL_FUSED and pl.workgroups == 256
    rc, pl = _plan(12, n_tokens=96, max_seg_len=8, r=64)
    assert rc == 0 and pl.kernel == sg.KERNEL_TILE
    rc, pl = _plan(6, n_tokens=96, max_seg_len=16, r=64)         # the tile kernel is out: per row up to 128 rows at 4096
    assert rc == 0 and pl.kernel == sg.KERNEL_FUSED and (pl.slices, pl.workgroups) == (2, 192)
    rc, pl = _plan(6, n_tokens=96, max_seg_len=16, r=64, h_out=11008)
    assert rc == 0 and pl.kernel == sg.KERNEL_MATRIX and pl.launches == 3
    rc, pl = _plan(39, n_tokens=96, max_seg_len=3, r=64, h_in=5120, h_out=5120)
    assert rc == 0 and pl.kernel == sg.KERNEL_MATRIX
    rc, pl = _plan(128, n_tokens=512, max_seg_len=4, r=64)
    assert rc == 0 and pl.kernel == sg.KERNEL_VECTOR
    # long segments: the MFMA kernels, three launches
    rc, pl = _plan(4, n_tokens=3450, max_seg_len=891)
    assert rc == 0 and pl.kernel == sg.KERNEL_MATRIX and pl.launches == 3
    # forced paths
    rc, pl = _plan(64, n_tokens=64, max_seg_len=1, path=sg.PATH_VECTOR)
    assert rc == 0 and pl.kernel == sg.KERNEL_VECTOR
    rc, pl = _plan(64, n_tokens=64, max_seg_len=1, path=sg.PATH_MATRIX)
    assert rc == 0 and pl.kernel == sg.KERNEL_MATRIX
    rc, pl = _plan(4, n_tokens=400, max_seg_len=100, path=sg.PATH_FUSED)
    assert rc == 0 and pl.kernel == sg.KERNEL_TILE and pl.workgroups == 8 * 4 * 7
    rc, pl = _plan(4, n_tokens=3450, max_seg_len=891, path=sg.PATH_FUSED)
    assert rc == 3                                   # unsupported: too many row blocks to be resident
    # a few long segments still fit one launch
    rc, pl = _plan(1, n_tokens=1024, max_seg_len=1024)
    assert rc == 0 and pl.kernel == sg.KERNEL_TILE and pl.slices == 4 and pl.workgroups == 256
    rc, pl = _plan(4, n_tokens=2048, max_seg_len=512)
    assert rc == 0 and pl.kernel == sg.KERNEL_MATRIX
    # nothing to do
    rc, pl = _plan(0, n_tokens=0)
    assert rc == 0 and pl.kernel == sg.KERNEL_NONE and pl.launches == 0


def test_workspace_bytes_multi():
    one = sg.sgmv_workspace_bytes(3450, 16)
    assert sg.sgmv_workspace_bytes_multi(3450, 16, 1) == one
    two, three, four = (sg.sgmv_workspace_bytes_multi(3450, 16, n) for n in (2, 3, 4))
    assert one < two < three == four and (two - one) == (three - two) and two % 256 == 0
    assert sg.sgmv_workspace_bytes_multi(0, 16, 3) == 0


def test_plan_shrink():
    """Stand-alone shrink of one-row segments: one launch, a workgroup per segment while A_i is small (or the
    batch beyond the hand-off's), else one launch with the hand-off, else two launches."""
    p = sg.make_problem(sg.F16, 4096, 4096, 16, 1, 64, workspace=FAKE, workspace_bytes=1 << 30, max_seg_len=1,
                        workspace_ready=1)
    rc, pl = sg.sgmv_plan_shrink(p, 64, check=False)     # A_i of 128 KB: no Split-K
    assert rc == 0 and pl.kernel == sg.KERNEL_WHOLE and (pl.launches, pl.slices, pl.workgroups) == (1, 1, 64)
    p.h_out = 0                                       # the output width plays no part
    rc, pl = sg.sgmv_plan_shrink(p, 64, check=False)
    assert rc == 0 and pl.kernel == sg.KERNEL_WHOLE
    p.workspace_ready = 0                             # nor does the workspace
    rc, pl = sg.sgmv_plan_shrink(p, 64, check=False)
    assert rc == 0 and pl.kernel == sg.KERNEL_WHOLE
    p.workspace_ready, p.r = 1, 64                    # A_i of 512 KB: Split-K with the hand-off ...
    rc, pl = sg.sgmv_plan_shrink(p, 64, check=False)
    assert rc == 0 and pl.kernel == sg.KERNEL_FUSED and (pl.launches, pl.slices, pl.workgroups) == (1, 4, 256)
    p.workspace_ready = 0                             # ... which needs the prepared workspace
    rc, pl = sg.sgmv_plan_shrink(p, 64, check=False)
    assert rc == 0 and pl.kernel == sg.KERNEL_VECTOR and pl.launches == 2
    p.workspace_ready, p.r, p.n_tokens = 1, 32, 256   # beyond the hand-off's batches: a workgroup per segment again ...
    rc, pl = sg.sgmv_plan_shrink(p, 256, check=False)
    assert rc == 0 and pl.kernel == sg.KERNEL_WHOLE and pl.workgroups == 256
    p.n_tokens = 1024                                 # ... up to about 100 MB of weights
    rc, pl = sg.sgmv_plan_shrink(p, 1024, check=False)
    assert rc == 0 and pl.kernel == sg.KERNEL_VECTOR and pl.launches == 2
    p.r, p.n_tokens, p.h_in = 16, 64, 4104            # A_i not a whole number of the kernel's steps
    rc, pl = sg.sgmv_plan_shrink(p, 64, check=False)
    assert rc == 0 and pl.kernel == sg.KERNEL_FUSED
    p.path = sg.PATH_WHOLE
    assert sg.sgmv_plan_shrink(p, 64, check=False)[0] == 3
    p.h_in = 4096
    rc, pl = sg.sgmv_plan_shrink(p, 64, check=False)
    assert rc == 0 and pl.kernel == sg.KERNEL_WHOLE
    p.path = sg.PATH_VECTOR
    rc, pl = sg.sgmv_plan_shrink(p, 64, check=False)
    assert rc == 0 and pl.kernel == sg.KERNEL_VECTOR
    p.path, p.max_seg_len, p.n_tokens = sg.PATH_AUTO, 300, 1200
    rc, pl = sg.sgmv_plan_shrink(p, 4, check=False)
    assert rc == 0 and pl.kernel == sg.KERNEL_MATRIX and pl.launches == 2
    # small batches of longer segments: one launch per ROW of the batch; with a small A_i a workgroup per row ...
    p.max_seg_len, p.n_tokens = 29, 64
    rc, pl = sg.sgmv_plan_shrink(p, 17, check=False)
    assert rc == 0 and pl.kernel == sg.KERNEL_WHOLE and (pl.launches, pl.slices, pl.workgroups) == (1, 1, 64)
    p.max_seg_len, p.n_tokens = 0, 500
    rc, pl = sg.sgmv_plan_shrink(p, 30, check=False)
    assert rc == 0 and pl.kernel == sg.KERNEL_WHOLE and pl.workgroups == 504
    p.n_tokens = 600
    rc, pl = sg.sgmv_plan_shrink(p, 30, check=False)
    assert rc == 0 and pl.kernel == sg.KERNEL_MATRIX and pl.launches == 2
    # ... with a larger one Split-K and the hand-off (64 rows at any rank, 128 up to rank 32)
    p.r, p.max_seg_len, p.n_tokens = 64, 29, 64
    rc, pl = sg.sgmv_plan_shrink(p, 17, check=False)
    assert rc == 0 and pl.kernel == sg.KERNEL_FUSED and (pl.launches, pl.slices, pl.workgroups) == (1, 4, 256)
    p.n_tokens = 200
    rc, pl = sg.sgmv_plan_shrink(p, 30, check=False)
    assert rc == 0 and pl.kernel != sg.KERNEL_FUSED and pl.launches == 2
    p.r = 32                                          # 256 KB: without Split-K where the hand-off's batches end
    rc, pl = sg.sgmv_plan_shrink(p, 30, check=False)
    assert rc == 0 and pl.kernel == sg.KERNEL_WHOLE and pl.workgroups == 200
    p.r, p.max_seg_len, p.n_tokens = 16, 300, 1200
    for path in (sg.PATH_FUSED, sg.PATH_ROWS):        # add-on kernels only
        p.path = path
        assert sg.sgmv_plan_shrink(p, 4, check=False)[0] == 3
    p.path = sg.PATH_WHOLE                            # as asked: a workgroup per row
    rc, pl = sg.sgmv_plan_shrink(p, 4, check=False)
    assert rc == 0 and pl.kernel == sg.KERNEL_WHOLE and pl.workgroups == 1200
    assert sg.lib.sgmv_plan_shrink(None, 4, None) == 1


def test_plan_multi_projection_shapes():
    # few enough workgroups for all projections side by side (two workgroups per unit)
    rc, pl = _plan(64, 2, n_tokens=64, max_seg_len=1)
    assert rc == 0 and pl.kernel == sg.KERNEL_MULTI_SIDE and pl.launches == 1
    assert pl.workgroups == 4 * 64 * 2
    # more: every workgroup walks the projections
    rc, pl = _plan(64, 3, n_tokens=64, max_seg_len=1)
    assert rc == 0 and pl.kernel == sg.KERNEL_MULTI_PIPELINED and pl.launches == 1
    assert pl.workgroups == 4 * 64
    rc, pl = _plan(16, 4, n_tokens=16, max_seg_len=1)
    assert rc == 0 and pl.kernel == sg.KERNEL_MULTI_SIDE and pl.workgroups == 8 * 16 * 4
    # segments of a few rows in a small batch: per row, the add-ons side by side in one launch
    rc, pl = _plan(8, 3, n_tokens=16, max_seg_len=2)
    assert rc == 0 and pl.kernel == sg.KERNEL_MULTI_SIDE and (pl.launches, pl.slices, pl.workgroups) == (1, 8, 8 * 16 * 3)
    rc, pl = _plan(39, 3, n_tokens=64, max_seg_len=5)
    assert rc == 0 and pl.kernel == sg.KERNEL_MULTI_SIDE and (pl.launches, pl.slices, pl.workgroups) == (1, 4, 4 * 64 * 3)
    # 128 rows, three add-ons: the joint tile launch while it keeps at least four slices
    rc, pl = _plan(16, 3, n_tokens=128, max_seg_len=8)
    assert rc == 0 and pl.kernel == sg.KERNEL_TILE and (pl.launches, pl.slices, pl.workgroups) == (1, 5, 5 * 16 * 3)
    rc, pl = _plan(64, 3, n_tokens=128, max_seg_len=2)
    assert rc == 0 and pl.kernel == sg.KERNEL_MULTI_SIDE and (pl.launches, pl.slices) == (1, 2)
    # the tile kernel when asked for: the add-ons side by side in one launch while their workgroups
    # are all resident together, with fewer slices each if need be ...
    rc, pl = _plan(8, 3, n_tokens=16, max_seg_len=2, path=sg.PATH_FUSED)
    assert rc == 0 and pl.kernel == sg.KERNEL_TILE and pl.launches == 1
    assert pl.slices == 8 and pl.workgroups == 8 * 8 * 3
    rc, pl = _plan(16, 3, n_tokens=64, max_seg_len=4, path=sg.PATH_FUSED)
    assert rc == 0 and pl.kernel == sg.KERNEL_TILE and pl.launches == 1
    assert pl.slices == 5 and pl.workgroups == 5 * 16 * 3
    # ... in groups where they do not all fit (here two, then the third by itself) ...
    rc, pl = _plan(39, 3, n_tokens=64, max_seg_len=5, path=sg.PATH_FUSED)
    assert rc == 0 and pl.kernel == sg.KERNEL_TILE and pl.launches == 2
    assert pl.slices * 39 * 2 <= 256 and pl.workgroups == pl.slices * 39 * 2
    # ... and one add-on after the other beyond that
    rc, pl = _plan(64, 3, n_tokens=128, max_seg_len=2, path=sg.PATH_FUSED)
    assert rc == 0 and pl.kernel == sg.KERNEL_TILE and pl.launches == 3
    # rank 64, long segments, 64 rows or more: the joint tile launch (a single add-on takes the MFMA kernels) ...
    rc, pl = _plan(8, 3, n_tokens=128, max_seg_len=16, r=64)
    assert rc == 0 and pl.kernel == sg.KERNEL_TILE and pl.launches == 1
    rc, pl = _plan(8, 1, n_tokens=128, max_seg_len=16, r=64, h_in=8192, h_out=8192)
    assert rc == 0 and pl.kernel == sg.KERNEL_MATRIX
    # ... except two add-ons at widths up to 4096, which run per row side by side
    rc, pl = _plan(8, 2, n_tokens=128, max_seg_len=16, r=64)
    assert rc == 0 and pl.kernel == sg.KERNEL_MULTI_SIDE and (pl.slices, pl.workgroups) == (2, 512)
    rc, pl = _plan(64, 9, n_tokens=64, max_seg_len=1)
    assert rc == 2
    rc, pl = _plan(64, 0, n_tokens=64, max_seg_len=1)
    assert rc == 2


def test_plan_expand():
    """Stand-alone expand: a workgroup per segment (or, small batches of longer segments, per row) and
    strip of columns, or the MFMA kernels for long segments with a workspace."""
    p = sg.make_problem(sg.F16, 4096, 4096, 16, 1, 64, workspace=FAKE, workspace_bytes=1 << 30, max_seg_len=1,
                        workspace_ready=1)
    rc, pl = sg.sgmv_plan_expand(p, 64, check=False)
    assert rc == 0 and pl.kernel == sg.KERNEL_VECTOR and pl.launches == 1 and pl.workgroups == pl.slices * 64
    p.h_in = 0                                        # the input width plays no part
    assert sg.sgmv_plan_expand(p, 64, check=False)[0] == 0
    p.max_seg_len = 29                                # 17 segments, 64 rows: per row (rows padded to eight)
    rc, pl = sg.sgmv_plan_expand(p, 17, check=False)
    assert rc == 0 and pl.kernel == sg.KERNEL_VECTOR and pl.launches == 1 and pl.workgroups == pl.slices * 64
    p.n_tokens = 61
    rc, pl = sg.sgmv_plan_expand(p, 17, check=False)
    assert rc == 0 and pl.workgroups == pl.slices * 64
    p.path = sg.PATH_VECTOR                           # as asked: per segment
    rc, pl = sg.sgmv_plan_expand(p, 17, check=False)
    assert rc == 0 and pl.kernel == sg.KERNEL_VECTOR and pl.workgroups == pl.slices * 17
    p.path, p.n_tokens, p.max_seg_len = sg.PATH_AUTO, 1200, 300
    rc, pl = sg.sgmv_plan_expand(p, 4, check=False)
    assert rc == 0 and pl.kernel == sg.KERNEL_MATRIX and pl.launches == 2
    p.workspace, p.workspace_bytes, p.workspace_ready = None, 0, 0   # no workspace: the vector kernel
    rc, pl = sg.sgmv_plan_expand(p, 4, check=False)
    assert rc == 0 and pl.kernel == sg.KERNEL_VECTOR
    for path in (sg.PATH_FUSED, sg.PATH_WHOLE, sg.PATH_ROWS):
        p.path = path
        assert sg.sgmv_plan_expand(p, 4, check=False)[0] == 3
    assert sg.lib.sgmv_plan_expand(None, 4, None) == 1
    # ranks 32 and 64: while the launch is small, the kernel whose waves divide the weight rows (strips of 512 columns)
    for r, n, strips in ((64, 64, 8), (32, 128, 8), (64, 192, 2), (16, 64, 4)):
        q = sg.make_problem(sg.F16, 4096, 4096, r, 1, n, max_seg_len=1)
        rc, pl = sg.sgmv_plan_expand(q, n, check=False)
        assert rc == 0 and pl.kernel == sg.KERNEL_VECTOR and pl.slices == strips, (r, n, pl.slices)
    q = sg.make_problem(sg.F16, 4096, 4096, 16, 1, 64, max_seg_len=1, expand_threads=512)
    assert sg.sgmv_plan_expand(q, 64, check=False)[0] == 3          # not below rank 32
    q = sg.make_problem(sg.F16, 4096, 4096, 64, 1, 1024, max_seg_len=1, expand_threads=512)
    rc, pl = sg.sgmv_plan_expand(q, 1024, check=False)
    assert rc == 0 and pl.slices == 8 and pl.workgroups == 8 * 1024


def test_plan_agrees_with_the_resource_limits():
    """Every single-launch plan keeps all its workgroups resident: at most 256 (one per
    compute unit), 512 for the side-by-side kernel, 768 for per-row launches; LDS within 160 KiB."""
    for r in (8, 16, 32, 64):
        for h_in, h_out in ((4096, 4096), (4096, 11008), (13824, 5120), (64, 64), (5120, 13824)):
            for n_segs, n_tokens, m in ((1, 1, 1), (7, 7, 1), (64, 64, 1), (200, 200, 1), (256, 256, 1),
                                        (3, 40, 16), (39, 64, 5), (64, 640, 29), (100, 300, 3), (2, 128, 64)):
                rc, pl = _plan(n_segs, r=r, h_in=h_in, h_out=h_out, n_tokens=n_tokens, max_seg_len=m)
                assert rc == 0
                if pl.kernel in (sg.KERNEL_FUSED, sg.KERNEL_TILE):
                    # (per-row launches of up to 384 rows: two slices each, three workgroups per unit)
                    most = 512 if m == 1 or pl.kernel == sg.KERNEL_TILE else 768
                    assert pl.launches == 1 and 0 < pl.workgroups <= most, (r, h_in, n_segs, pl.workgroups)
                    if pl.kernel == sg.KERNEL_TILE:
                        assert pl.workgroups <= 256 and pl.lds_bytes <= 160 * 1024
                elif pl.kernel == sg.KERNEL_WHOLE:   # its workgroups never wait for each other: any grid
                    assert pl.launches == 1 and pl.lds_bytes == 0 and (m == 1 or h_in * r <= 32768)   # longer segments: per row, small A_i
                else:
                    assert pl.kernel in (sg.KERNEL_VECTOR, sg.KERNEL_MATRIX)


def test_plan_tile_needs_resident_workgroups_and_lds():
    # 32 segments of up to 64 rows: four row blocks per segment leave two slices, whose weight
    # slices do not fit the LDS: the launch-per-step kernels take the call
    rc, pl = _plan(32, n_tokens=248, max_seg_len=64, r=32)
    assert rc == 0 and pl.kernel == sg.KERNEL_MATRIX
    rc, pl = _plan(32, n_tokens=248, max_seg_len=64)          # up to rank 16 and 256 rows: per row
    assert rc == 0 and pl.kernel == sg.KERNEL_FUSED and (pl.slices, pl.workgroups) == (2, 496)
    # a forced slice count that cannot be resident is not taken by the single-launch kernels
    rc, pl = _plan(64, n_tokens=640, max_seg_len=29, ksplit=8, path=sg.PATH_FUSED)
    assert rc == 3


def test_plan_tile_counts_only_row_blocks_with_rows():
    # 17 segments, the longest of 29 rows (two row blocks): 34 blocks in the grid, but at most
    # 17 + 64/16 = 21 hold rows, so eight slices are resident (8 * 21 <= 256) in a grid of 272
    rc, pl = _plan(17, n_tokens=64, max_seg_len=29, path=sg.PATH_FUSED)
    assert rc == 0 and pl.kernel == sg.KERNEL_TILE and (pl.slices, pl.workgroups) == (8, 272)
    # a grid far beyond one workgroup per compute unit is not taken
    rc, pl = _plan(8, n_tokens=1000, max_seg_len=300)
    assert rc == 0 and pl.kernel == sg.KERNEL_MATRIX


def test_plan_sixteen_slices_for_small_batches_at_high_rank():
    # a slice of A_i at eight slices would take more than one batch of loads: sixteen slices
    for kw, S in ((dict(r=64), 16), (dict(r=64, h_in=5120, h_out=5120), 16), (dict(r=32, h_in=5120, h_out=5120), 16),
                  (dict(r=32), 8), (dict(r=16), 8)):
        rc, pl = _plan(4, n_tokens=4, max_seg_len=1, **kw)
        assert rc == 0 and pl.kernel == sg.KERNEL_FUSED and pl.slices == S, (kw, pl.slices)
    rc, pl = _plan(16, n_tokens=16, max_seg_len=1, r=64)
    assert rc == 0 and (pl.slices, pl.workgroups) == (16, 256)
    rc, pl = _plan(32, n_tokens=32, max_seg_len=1, r=64)      # 512 workgroups would not be resident
    assert rc == 0 and pl.slices == 8


def test_plan_multi_at_width_5120():
    # four slices of 1280 features are too deep for the pipelined kernel: three projections of 64
    # segments run side by side (768 workgroups, three per compute unit); rank 64 runs them in turn
    rc, pl = _plan(64, 3, n_tokens=64, max_seg_len=1, h_in=5120, h_out=5120)
    assert rc == 0 and pl.kernel == sg.KERNEL_MULTI_SIDE and pl.workgroups == 768 and pl.launches == 1
    rc, pl = _plan(64, 3, n_tokens=64, max_seg_len=1, h_in=5120, h_out=5120, r=64)
    assert rc == 0 and pl.kernel == sg.KERNEL_FUSED and pl.launches == 3


def test_static_entry_point_rejects_before_touching_a_device():
    # the size limit and the plain argument errors are decided on the host
    big = sg.make_problem(sg.F16, 256, 256, 64, 1, 4096, max_seg_len=1)
    assert sg.sgmv_workspace_bytes(4096, 64) > sg.STATIC_MAX_WORKSPACE_BYTES
    assert sg.sgmv_add_lora_static(big, 16, 16, 16, 16, 16, 4, 0, 1.0, check=False) == 5     # too large
    small = sg.make_problem(sg.F16, 256, 256, 16, 1, 4, max_seg_len=1)
    assert sg.sgmv_add_lora_static(small, None, 16, 16, 16, 16, 4, 0, 1.0, check=False) == 1  # y is NULL
    assert sg.sgmv_add_lora_static(small, 24, 16, 16, 16, 16, 4, 0, 1.0, check=False) == 4    # y misaligned
    assert sg.sgmv_add_lora_static(small, 16, 16, 16, 16, 16, 4, 3, 1.0, check=False) == 6    # layer out of range
    assert sg.sgmv_add_lora_static(small, 16, 16, 16, 16, 16, 0, 0, 1.0, check=False) == 0    # nothing to do
    assert sg.STATIC_SCRATCH_BYTES == 9 << 20
