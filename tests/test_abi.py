"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and reports argument errors before touching the device."""
import ctypes
import os
import re

import pytest

import paper_2506_08889_amd as seer
from paper_2506_08889_amd.api import _KVLayout

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "seer.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(seer_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = seer.load_library()
    names = declared_symbols()
    assert {"seer_gate_select", "seer_sparse_decode", "seer_dense_decode", "seer_gate_workspace_bytes",
            "seer_decode_workspace_bytes", "seer_status_string", "seer_version"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"libseer.so does not export {n}"
    assert seer.version() >= 100


def test_status_strings():
    lib = seer.load_library()
    seen = set()
    for code in range(0, -8, -1):
        s = lib.seer_status_string(code).decode()
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 8
    assert lib.seer_status_string(-99).decode() == "unknown status"


def test_workspace_queries():
    assert seer.gate_workspace_bytes(64, 8, 2048) >= 64 * 8 * 2048 * 8
    n = seer.decode_workspace_bytes(64, 40, 8, 128, 205)
    assert n > 0 and n % 256 == 0
    with pytest.raises(seer.SeerError) as e:
        seer.decode_workspace_bytes(1, 7, 2, 128, 16)       # Hq not a multiple of Hkv
    assert e.value.status == -2
    with pytest.raises(seer.SeerError) as e:
        seer.decode_workspace_bytes(1, 8, 2, 64, 16)        # head dim 64 is not built
    assert e.value.status == -3
    with pytest.raises(seer.SeerError) as e:
        seer.decode_workspace_bytes(1, 34, 2, 128, 16)      # 17 query rows per kv head (16 = tokens x heads is the cap)
    assert e.value.status == -3
    with pytest.raises(seer.SeerError):
        seer.gate_workspace_bytes(0, 8, 16)


def test_argument_errors_are_reported_before_any_launch():
    """Fake, never-dereferenced device addresses: every call below must fail in validation."""
    lib = seer.load_library()
    P = ctypes.c_void_p(0x10000)
    lay = _KVLayout()
    lay.k, lay.v = 0x10000, 0x20000
    lay.stride_seq, lay.stride_head, lay.stride_token = 8 * 1024 * 128, 1024 * 128, 128
    lay.page_table, lay.max_pages, lay.page_size = None, 0, 0
    f = ctypes.c_float(0.1)

    def sparse(q=P, layp=ctypes.byref(lay), sl=P, bi=P, nk=P, max_sel=16, B=1, Hq=8, Hkv=2, d=128, bs=64,
               out=P, dt=0, lse=P, ws=P, wsb=1 << 30, hints=0):
        return lib.seer_sparse_decode(q, layp, sl, bi, nk, max_sel, B, Hq, Hkv, d, bs, f, out, dt, lse, ws, wsb, hints,
                                      None)

    assert sparse(q=None) == -1
    assert sparse(bi=None) == -1
    assert sparse(out=None) == -1
    assert sparse(layp=None) == -1
    assert sparse(Hq=7) == -2
    assert sparse(B=0) == -2
    assert sparse(d=64) == -3
    assert sparse(bs=48) == -3
    assert sparse(Hq=18) == -3
    assert sparse(dt=5) == -3
    assert sparse(hints=2) == -3                                 # unknown hint bit
    assert sparse(ws=None) == -4
    assert sparse(wsb=16) == -4
    assert sparse(ws=ctypes.c_void_p(0x10008)) == -4            # misaligned workspace
    assert sparse(q=ctypes.c_void_p(0x10004)) == -2              # misaligned q
    lay.stride_token = 100
    assert sparse() == -2
    lay.stride_token = 128
    lay.page_table, lay.max_pages, lay.page_size = 0x30000, 4, 96   # page not a multiple of the block
    assert sparse() == -2
    lay.page_table, lay.max_pages, lay.page_size = None, 0, 0

    assert lib.seer_dense_decode(P, ctypes.byref(lay), P, 0, 1, 8, 2, 128, 64, f, P, 0, P, P, 1 << 30, 0, None) == -2
    assert lib.seer_dense_decode(None, ctypes.byref(lay), P, 4, 1, 8, 2, 128, 64, f, P, 0, P, P, 1 << 30, 0, None) == -1

    def gate(qg=P, kc=P, sl=P, B=1, Hkv=2, Dg=128, nb_max=64, bs=64, mode=0, budget=1024, bb=None, thr=0.0,
             bi=P, nk=P, max_sel=16, ws=P, wsb=1 << 30, sj=128, hints=0):
        return lib.seer_gate_select(qg, kc, 2 * 64 * 128, 64 * 128, sj, sl, B, Hkv, Dg, nb_max, bs, mode, budget,
                                    bb, thr, bi, nk, max_sel, ws, wsb, hints, None)

    assert gate(qg=None) == -1
    assert gate(nk=None) == -1
    assert gate(Dg=64) == -3
    assert gate(mode=3) == -3
    assert gate(hints=4) == -3
    assert gate(mode=2, max_sel=16) == -5              # top-p may select every block too
    assert gate(bs=100) == -3
    assert gate(budget=-5) == -2
    assert gate(sj=64) == -2
    assert gate(max_sel=8) == -5                       # 1024 tokens = 16 blocks do not fit 8 slots
    assert gate(mode=1, max_sel=16) == -5              # threshold mode may select every block
    assert gate(mode=1, max_sel=64, thr=float("nan")) == -2
    assert gate(ws=None) == -4
    assert gate(wsb=8) == -4


def test_gate_select_q_argument_errors_come_before_the_gate_query_kernel():
    """The one-call gate validates the arguments of both of its halves before launching the first."""
    lib = seer.load_library()
    P = ctypes.c_void_p(0x10000)

    def call(qn=P, wq=P, cos=P, sin=P, kc=P, sl=P, B=2, Hq=8, Hkv=2, d=128, Dg=128, nb_max=64, bs=64, mode=0, budget=1024,
             thr=0.0, bi=P, nk=P, max_sel=16, ws=P, wsb=1 << 30, hints=0):
        return lib.seer_gate_select_q(qn, wq, cos, sin, 4097, kc, 2 * 64 * 128, 64 * 128, 128, sl, B, Hq, Hkv, d, Dg, nb_max,
                                      bs, mode, budget, None, thr, bi, nk, max_sel, None, ws, wsb, hints, None)

    assert call(ws=None) == -4 and call(wsb=64) == -4
    assert call(kc=None) == -1 and call(nk=None) == -1
    assert call(bs=48) == -3 and call(mode=7) == -3 and call(hints=2) == -3
    assert call(max_sel=8) == -5 and call(mode=1, max_sel=16) == -5
    assert call(budget=-1) == -2
    assert call(qn=None) == -1 and call(wq=None) == -1 and call(cos=None) == -1      # the query half's own checks
    assert call(Hq=7) == -2 and call(d=64) == -3


def test_knobs_roundtrip():
    for knob, vals in ((0, (1, 2, 0)), (1, (3, 17, 0)), (3, (1, 2, 0))):
        for v in vals:
            seer.set_knob(knob, v)
            assert seer.get_knob(knob) == v
    with pytest.raises(seer.SeerError):
        seer.set_knob(0, 9)
    with pytest.raises(seer.SeerError):
        seer.set_knob(42, 1)
    with pytest.raises(seer.SeerError):
        seer.set_knob(2, 1)          # what a caller knows about its lists travels with the call (hints), not a knob


def test_split_plan_properties_on_the_host():
    """The planner is host logic: whatever the sizes and knobs, the slices cover the list capacity,
    a slice holds at least 4 entries (or the whole list), there are at most 256 slices, and the plan
    never needs more workspace than the size query hands out."""
    import itertools
    for knob in (0, 1, 3):
        seer.set_knob(knob, 0)
    try:
        for ragged, forced in itertools.product((0, 1), (0, 1, 3, 64, 1000)):
            seer.set_knob(1, forced)
            for B, Hkv, nb, bs in itertools.product((1, 4, 16, 32, 64, 300), (1, 2, 8), (1, 3, 13, 64, 205, 2048, 5000),
                                                    (16, 64, 128)):
                ns, per = seer.decode_plan(B, Hkv, nb, bs, ragged=bool(ragged))
                assert 1 <= ns <= 256 and per >= 1
                assert ns * per >= nb and (ns - 1) * per < nb          # covers the list, no empty last slice
                assert per >= min(4, nb) or ns == 1
                if forced and not ragged:
                    assert ns <= forced
        seer.set_knob(1, 0)
        # equal-length lists: no cut when there are at least as many groups as compute units, and short
        # lists stay whole when cutting saves less than a merge launch
        assert seer.decode_plan(64, 8, 205, 64) == (1, 205)
        assert seer.decode_plan(32, 8, 51, 64)[0] == 1
        assert seer.decode_plan(16, 8, 13, 64)[0] == 1
        assert seer.decode_plan(16, 8, 64, 64)[0] == 2
        assert seer.decode_plan(1, 8, 256, 64)[0] == 32
        # lists of very different lengths: slices of about 2048 tokens, shorter when the whole batch holds
        # only a few slices per resident work-group
        assert seer.decode_plan(128, 8, 203, 64, ragged=True) == (7, 29)
        assert seer.decode_plan(128, 8, 2022, 64, ragged=True) == (64, 32)
        assert seer.decode_plan(32, 8, 49, 128, ragged=True) == (7, 7)
        assert seer.decode_plan(64, 8, 205, 64, ragged=True)[1] * 64 <= 2048
    finally:
        for knob in (0, 1, 3):
            seer.set_knob(knob, 0)
    with pytest.raises(seer.SeerError):
        seer.decode_plan(0, 8, 16, 64)
    with pytest.raises(seer.SeerError):
        seer.decode_plan(1, 8, 16, 48)


def test_training_forward_argument_errors_on_the_host():
    lib = seer.load_library()
    n = seer.attn_ground_truth_workspace_bytes(1, 1000, 8, 2, 128, 64)
    # block maxima only for the rows that can see a block: sum over the 16 blocks of (1008 - 64 j) rows per head
    tri = sum(1008 - 64 * j for j in range(16))
    assert n >= 8 * tri * 4 + 8 * 1000 * 4 and n % 256 == 0
    assert n < 8 * 16 * 1008 * 4          # well below the full rows-by-blocks rectangle
    for bad in ((0, 64, 8, 2, 128, 64), (1, 0, 8, 2, 128, 64), (1, 64, 7, 2, 128, 64)):
        with pytest.raises(seer.SeerError) as e:
            seer.attn_ground_truth_workspace_bytes(*bad)
        assert e.value.status == -2
    for bad in ((1, 64, 8, 2, 64, 64), (1, 64, 8, 2, 128, 48), (1, 64, 18, 2, 128, 64)):
        with pytest.raises(seer.SeerError) as e:
            seer.attn_ground_truth_workspace_bytes(*bad)
        assert e.value.status == -3
    import ctypes
    from paper_2506_08889_amd.api import _KVLayout
    P = ctypes.c_void_p(4096)
    lay = _KVLayout()
    lay.k, lay.v = 4096, 8192
    lay.stride_seq, lay.stride_head, lay.stride_token = 2 * 64 * 128, 64 * 128, 128

    def call(q=P, B=1, T=64, Hq=8, Hkv=2, d=128, bs=64, scale=0.1, out=P, gt=P, ws=P, wsb=1 << 30, layout=lay):
        return lib.seer_attn_ground_truth(q, ctypes.byref(layout), None, B, T, Hq, Hkv, d, bs, ctypes.c_float(scale),
                                          out, 0, None, gt, ws, wsb, None)
    assert call(q=None) == -1 and call(gt=None) == -1
    assert call(T=0) == -2 and call(Hq=7) == -2
    assert call(bs=48) == -3 and call(scale=0.0) == -3 and call(scale=-1.0) == -3
    assert call(ws=None) == -4 and call(wsb=1024) == -4
    paged = _KVLayout()
    paged.k, paged.v = 4096, 8192
    paged.stride_seq, paged.stride_head, paged.stride_token = 2 * 64 * 128, 64 * 128, 128
    paged.page_table, paged.max_pages, paged.page_size = 4096, 1, 64
    assert call(layout=paged) == -3


def test_bench_refuses_more_than_one_gpu():
    """bench.py runs on one GPU; asked for more it exits with a message that says so (no GPU needed)."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and "--gpus must be 1" in r.stderr
