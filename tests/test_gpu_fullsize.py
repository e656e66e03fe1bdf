"""GPU parity at the FULL sizes of the benchmark configurations, in the launch configuration
bench.py times (default knobs, bf16 output, caller-provided workspaces): every block index of
every group against the oracle (bit-exact), and the decode output on a sample of (sequence,
kv-head) groups that always includes the first and the last group."""
import numpy as np
import pytest
import torch

import oracle
import paper_2506_08889_amd as seer
import synth
from helpers import (check_decode, check_indices, gather_groups, oracle_decode_on_groups, oracle_gate,
                     pick_threshold)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def sample_groups(G, n, seed):
    rng = np.random.default_rng(seed)
    inner = rng.choice(np.arange(1, G - 1), size=min(n, G) - 2, replace=False) if G > 2 else np.array([], dtype=int)
    return np.sort(np.concatenate([[0, G - 1], inner]).astype(np.int64))


def run_full(name, n_sample, mode=seer.SELECT_TOPK, keep=None, block_size=None):
    for k in (0, 1, 3):
        seer.set_knob(k, 0)
    w = synth.CONFIGS[name]
    seer.set_knob(2, 1 if (w.seqlen_dist != "fixed" or w.budget_tokens == 0) else 0)   # as bench.py does
    if block_size:
        w = synth.scaled(w, block_size=block_size)
    print(f"[full] {w.name} b={w.block_size} mode={mode}", flush=True)
    inp = synth.make_inputs(w, DEV)
    max_sel, thr = inp.max_sel, 0.0
    if mode == seer.SELECT_THRESHOLD:
        _, _, scores = oracle_gate(inp, return_scores=True)
        thr = pick_threshold(scores, inp.seqlens_cpu, w.block_size, w.Dg, keep)
        max_sel = inp.nb_max
    ref_idx, ref_cnt = oracle_gate(inp, mode=mode, threshold=thr, max_sel=max_sel)
    idx, cnt = seer.gate_select(inp.q_gate, inp.kc, inp.seqlens, w.block_size, mode=mode,
                                budget_tokens=w.budget_tokens, budget_blocks=inp.budget_blocks, threshold=thr,
                                max_sel=max_sel)
    torch.cuda.synchronize()
    check_indices(idx, cnt, ref_idx, ref_cnt, what=f"{w.name} gate (all {w.B * w.Hkv} groups)")
    out, lse = seer.sparse_decode(inp.q, inp.k, inp.v, inp.seqlens, idx, cnt, w.block_size, w.scale,
                                  page_table=inp.page_table, page_size=inp.page_size)
    torch.cuda.synchronize()
    groups = sample_groups(w.B * w.Hkv, n_sample, w.seed)
    print(f"[full] {w.name}: oracle decode on {len(groups)} groups", flush=True)
    ro, rl = oracle_decode_on_groups(inp, ref_idx, ref_cnt, groups)
    go = gather_groups(out, w, groups, w.g)
    gl = gather_groups(lse, w, groups, w.g)
    check_decode(go, gl, ro, rl, tight=False, what=f"{w.name} decode sample")
    # whole output: finite, and rows of non-empty groups are not all zero
    assert torch.isfinite(out.float()).all() and torch.isfinite(lse).all()
    return inp, idx, cnt


def test_c2_full_size():
    run_full("c2", 128)


def test_c3_full_size_paged():
    run_full("c3", 48)


def test_c4_full_size_headline():
    inp, idx, cnt = run_full("c4", 24)
    # the dense flash-decode of the same shape, on a few groups
    w = inp.w
    out, lse = seer.dense_decode(inp.q, inp.k, inp.v, inp.seqlens, inp.nb_max, w.block_size, w.scale)
    torch.cuda.synchronize()
    groups = np.array([0, 257, w.B * w.Hkv - 1])
    ro, rl = oracle_decode_on_groups(inp, None, None, groups) if False else (None, None)
    # dense oracle: every block listed
    nb = inp.nb_max
    all_idx = torch.arange(nb, dtype=torch.int32).expand(w.B, w.Hkv, nb).contiguous()
    all_cnt = torch.full((w.B, w.Hkv), nb, dtype=torch.int32)
    ro, rl = oracle_decode_on_groups(inp, all_idx, all_cnt, groups)
    check_decode(gather_groups(out, w, groups, w.g), gather_groups(lse, w, groups, w.g), ro, rl, tight=False,
                 what="c4 dense sample")


@pytest.mark.parametrize("bs", [64, 128])
def test_c5_full_size_topk(bs):
    run_full("c5", 32, block_size=bs)


def test_c5_full_size_threshold_90pct():
    run_full("c5", 32, mode=seer.SELECT_THRESHOLD, keep=0.10)
