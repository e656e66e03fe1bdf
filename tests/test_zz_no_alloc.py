"""seer_sparse_decode_noalloc: the entry point for callers that cannot allocate (the split-K partials
live in a scratch array inside the library image).  It must return what seer_sparse_decode returns -
checked bit for bit against that call and, to the parity bars, against the fp64 oracle - on two calls
in a row, the second on a smaller input that leaves most of the first call's partials in the array."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2506_08889_amd as seer
import synth
from paper_2506_08889_amd.api import _KVLayout

DEV = "cuda:0"


def test_noalloc_sizes_beyond_the_scratch_are_refused_on_the_host():
    """No GPU needed: fake, never-dereferenced addresses; the size check comes before any device work."""
    lib = seer.load_library()
    P = ctypes.c_void_p(0x10000)
    lay = _KVLayout()
    lay.k, lay.v = 0x10000, 0x20000
    lay.stride_seq, lay.stride_head, lay.stride_token = 8 * 4096 * 128, 4096 * 128, 128
    lay.page_table, lay.max_pages, lay.page_size = None, 0, 0
    f = ctypes.c_float(0.1)

    def call(q=P, B=4096, Hq=32, Hkv=8, max_sel=2048, hints=seer.HINT_RAGGED_LISTS, out=P):
        return lib.seer_sparse_decode_noalloc(q, ctypes.byref(lay), P, P, P, max_sel, B, Hq, Hkv, 128, 64, f, out, 0, P,
                                              hints, None)

    ns, _ = seer.decode_plan(4096, 8, 2048, 64, ragged=True)
    assert 4096 * 8 * ns * 4 * 520 > seer.NOALLOC_SCRATCH_BYTES           # this plan's partials do not fit
    assert call() == -7
    assert "scratch" in lib.seer_status_string(-7).decode()
    assert call(q=None) == -1 and call(out=None) == -1                     # the usual validation still comes first
    assert call(Hq=33) == -2 and call(hints=8) == -3


@pytest.mark.gpu
def test_noalloc_matches_the_workspace_entry_point_on_two_calls_in_a_row():
    from helpers import check_decode, oracle_decode
    for k in (0, 1, 3):
        seer.set_knob(k, 0)
    results = []
    # second case: fewer sequences, shorter lists, fewer slices - it overwrites only part of what the first left
    for case, (B, S, k_sel) in enumerate(((5, 64 * 90 + 13, 48), (2, 64 * 30 + 40, 20))):
        w = synth.Workload(f"noalloc{case}", B=B, Hq=8, Hkv=2, block_size=64, seqlen=S, budget_tokens=64 * k_sel,
                           seed=880 + case)
        print(f"[noalloc] case {case}: B={B} S={S} lists of {k_sel}", flush=True)
        inp = synth.make_inputs(w, DEV)
        nb = (inp.seqlens_cpu + 63) // 64
        idx, cnt = synth.random_block_lists(B, 2, nb, [k_sel] * B, k_sel, torch.Generator().manual_seed(case), ascending=False)
        idx[:, :, 0] = int(nb[0]) - 1                                     # the partial last block is listed
        for i in range(B):
            for h in range(2):
                dup = (idx[i, h, 1:] == int(nb[0]) - 1).nonzero()
                if len(dup):
                    idx[i, h, 1 + int(dup[0])] = -1                       # keep it listed once (invalid entries are skipped)
        ns, per = seer.decode_plan(B, 2, k_sel, 64)
        assert ns > 1, "the case must really use the scratch (several slices + merge)"
        d_idx, d_cnt = idx.to(DEV), cnt.to(DEV)
        ref_out, ref_lse = oracle_decode(inp, idx, cnt)
        for dt, tight in ((torch.float32, True), (torch.bfloat16, False)):
            want_out, want_lse = seer.sparse_decode(inp.q, inp.k, inp.v, inp.seqlens, d_idx, d_cnt, 64, w.scale, out_dtype=dt)
            out = torch.full((B, 8, 128), 9.0, dtype=dt, device=DEV)
            lse = torch.full((B, 8), 9.0, dtype=torch.float32, device=DEV)
            torch.cuda.synchronize()
            seer.sparse_decode_noalloc(inp.q, inp.k, inp.v, inp.seqlens, d_idx, d_cnt, 64, w.scale, out=out, lse=lse)
            torch.cuda.synchronize()
            assert torch.equal(out, want_out) and torch.equal(lse, want_lse), f"case {case} {dt}: differs from seer_sparse_decode"
            check_decode(out, lse, ref_out, ref_lse, tight=tight, what=f"noalloc case {case} {dt}")
            # the plan for lists of very different lengths keeps its hand-out word in the same array
            out.fill_(9.0); lse.fill_(9.0)
            seer.sparse_decode_noalloc(inp.q, inp.k, inp.v, inp.seqlens, d_idx, d_cnt, 64, w.scale, out=out, lse=lse, ragged=True)
            torch.cuda.synchronize()
            check_decode(out, lse, ref_out, ref_lse, tight=tight, what=f"noalloc ragged case {case} {dt}")
        results.append((out, lse))
    # a single slice (no partials at all) goes through the same entry point
    seer.set_knob(1, 1)
    try:
        out1 = torch.empty(2, 8, 128, dtype=torch.float32, device=DEV)
        lse1 = torch.empty(2, 8, dtype=torch.float32, device=DEV)
        seer.sparse_decode_noalloc(inp.q, inp.k, inp.v, inp.seqlens, d_idx, d_cnt, 64, w.scale, out=out1, lse=lse1)
        torch.cuda.synchronize()
        check_decode(out1, lse1, ref_out, ref_lse, tight=True, what="noalloc single slice")
    finally:
        seer.set_knob(1, 0)
