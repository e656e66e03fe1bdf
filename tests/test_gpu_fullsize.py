"""GPU parity at the FULL sizes of the benchmark configurations, in the launch configuration
bench.py times (default knobs, the same per-call hints, caller-provided workspaces): every block
index of every group against the oracle (bit-exact), and the decode output on a sample of (sequence,
kv-head) groups that always includes the first and the last group - once with bf16 output at the
contract's bars and once with fp32 output at the tight bars of tests/helpers.py, which a dropped block
or tail token cannot pass."""
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


def is_ragged(w, mode):
    """The hint bench.py passes: lists of very different lengths."""
    return w.seqlen_dist != "fixed" or w.budget_tokens == 0 or mode != seer.SELECT_TOPK


def gate_and_decode_full(inp, n_sample, mode=seer.SELECT_TOPK, keep=None, scores=None, host_kv=None, what=""):
    """Gate on every group (bit-exact), decode on the whole batch, oracle decode on a sample."""
    w = inp.w
    for k in (0, 1, 3):
        seer.set_knob(k, 0)
    ragged = is_ragged(w, mode)
    max_sel, thr = inp.max_sel, 0.0
    if mode == seer.SELECT_THRESHOLD:
        thr = pick_threshold(scores, inp.seqlens_cpu, w.block_size, w.Dg, keep)
        max_sel = inp.nb_max
    print(f"[full] {what}: gate, {w.B * w.Hkv} groups, mode={mode} keep={keep} max_sel={max_sel}", flush=True)
    ref_idx, ref_cnt = oracle_gate(inp, mode=mode, threshold=thr, max_sel=max_sel)
    idx, cnt = seer.gate_select(inp.q_gate, inp.kc, inp.seqlens, w.block_size, mode=mode,
                                budget_tokens=w.budget_tokens, budget_blocks=inp.budget_blocks, threshold=thr,
                                max_sel=max_sel, ragged=ragged)
    torch.cuda.synchronize()
    check_indices(idx, cnt, ref_idx, ref_cnt, what=f"{what} gate (all {w.B * w.Hkv} groups)")
    groups = sample_groups(w.B * w.Hkv, n_sample, w.seed)
    print(f"[full] {what}: oracle decode on {len(groups)} groups, {int(ref_cnt.sum())} blocks selected in all", flush=True)
    ro, rl = oracle_decode_on_groups(inp, ref_idx, ref_cnt, groups, host_kv=host_kv)
    for dt, tight in ((torch.bfloat16, False), (torch.float32, True)):
        out, lse = seer.sparse_decode(inp.q, inp.k, inp.v, inp.seqlens, idx, cnt, w.block_size, w.scale,
                                      page_table=inp.page_table, page_size=inp.page_size, out_dtype=dt, ragged=ragged)
        torch.cuda.synchronize()
        check_decode(gather_groups(out, w, groups, w.g), gather_groups(lse, w, groups, w.g), ro, rl, tight=tight,
                     what=f"{what} decode sample {dt}")
        # whole output finite; lse is -inf exactly for the groups that selected nothing
        assert torch.isfinite(out.float()).all()
        empty = (cnt == 0).repeat_interleave(w.g, dim=1)
        assert torch.equal(torch.isneginf(lse), empty) and torch.isfinite(lse[~empty]).all()
    return idx, cnt


def run_full(name, n_sample, **kw):
    w = synth.CONFIGS[name]
    print(f"[full] {w.name} b={w.block_size}: inputs", flush=True)
    inp = synth.make_inputs(w, DEV)
    idx, cnt = gate_and_decode_full(inp, n_sample, what=w.name, **kw)
    return inp, idx, cnt


def test_c2_full_size():
    run_full("c2", 128)


def test_c3_full_size_paged():
    run_full("c3", 48)


@pytest.mark.timeout(600)
def test_c4_full_size_headline():
    """The headline configuration: 64 sampled groups of 512 (first and last included), bf16 output at
    the contract's bars and fp32 output at the tight ones; then the dense flash-decode of the same shape."""
    inp, idx, cnt = run_full("c4", 64)
    w = inp.w
    groups = np.array([0, 257, w.B * w.Hkv - 1])
    nb = inp.nb_max
    all_idx = torch.arange(nb, dtype=torch.int32).expand(w.B, w.Hkv, nb).contiguous()
    all_cnt = torch.full((w.B, w.Hkv), nb, dtype=torch.int32)
    print("[full] c4: dense oracle on 3 groups", flush=True)
    ro, rl = oracle_decode_on_groups(inp, all_idx, all_cnt, groups)
    for dt, tight in ((torch.bfloat16, False), (torch.float32, True)):
        out, lse = seer.dense_decode(inp.q, inp.k, inp.v, inp.seqlens, inp.nb_max, w.block_size, w.scale, out_dtype=dt)
        torch.cuda.synchronize()
        check_decode(gather_groups(out, w, groups, w.g), gather_groups(lse, w, groups, w.g), ro, rl, tight=tight,
                     what=f"c4 dense sample {dt}")


@pytest.mark.timeout(900)
@pytest.mark.parametrize("bs", [64, 128])
def test_c5_full_size_sweep_topk_and_threshold(bs):
    """Batch 128, log-uniform lengths, paged: token-budget and threshold selection at 50 / 75 / 90 / 95 %
    sparsity.  One set of tensors per block size (the draws do not depend on the budget); indices of all
    1024 groups, decode on 32 sampled groups per point."""
    w = synth.scaled(synth.CONFIGS["c5"], block_size=bs)
    print(f"[full] c5 b={bs}: inputs", flush=True)
    inp = synth.make_inputs(w, DEV)
    host_kv = {}                                   # host copies of the sampled heads' page pools, made once
    _, _, scores = oracle_gate(inp, return_scores=True)
    for keep in (0.5, 0.25, 0.10, 0.05):
        inp.w = synth.scaled(w, budget_frac=keep)
        inp.budget_blocks_cpu = synth.block_budgets(inp.seqlens_cpu, bs, keep)
        inp.budget_blocks = inp.budget_blocks_cpu.to(DEV)
        inp.max_sel = int(inp.budget_blocks_cpu.max())
        gate_and_decode_full(inp, 32, host_kv=host_kv, what=f"c5 b={bs} top-k keep={keep}")
        gate_and_decode_full(inp, 32, mode=seer.SELECT_THRESHOLD, keep=keep, scores=scores, host_kv=host_kv,
                             what=f"c5 b={bs} threshold keep={keep}")


def test_training_forward_long_sequence_every_row():
    """8192 tokens (64 query tiles x up to 128 key tiles), one group of two heads: every row of
    out / lse / ground truth against the oracle."""
    print("[full] training forward T=8192", flush=True)
    gen = synth.generator(DEV, 77)
    T, b = 8192, 64
    q = synth.randn_bf16((1, T, 2, 128), DEV, gen)
    k = synth.randn_bf16((1, 1, T, 128), DEV, gen)
    v = synth.randn_bf16((1, 1, T, 128), DEV, gen)
    out, lse, gt = seer.attn_ground_truth(q, k, v, b, 128 ** -0.5)
    torch.cuda.synchronize()
    ro, rl, rg = oracle.attn_ground_truth(q.cpu(), k.cpu(), v.cpu(), b, 128 ** -0.5)
    np.testing.assert_allclose(lse.cpu().numpy(), rl, rtol=0, atol=1e-3)
    np.testing.assert_allclose(gt.cpu().numpy(), rg, rtol=2e-4, atol=1e-7)
    err = np.abs(out.float().cpu().numpy() - ro)
    assert err.max() <= 1e-2 and (err.max(-1) <= 1e-2 * np.maximum(np.abs(ro).max(-1), 0.05) + 1e-6).all()


def test_training_forward_in_the_bench_configuration_on_sampled_rows():
    """The shape bench.py times (16384 tokens, c4's 40 / 8 heads, bf16 out): the first 512 rows against
    the oracle run on that prefix (causality makes them independent of the rest), late rows' out / lse
    against the decode oracle, and the properties every ground-truth row has."""
    print("[full] training forward T=16384, 40/8 heads", flush=True)
    w = synth.CONFIGS["c4"]
    gen = synth.generator(DEV, w.seed + 4000)
    T, b, Hq, Hkv = 16384, w.block_size, w.Hq, w.Hkv
    q = synth.randn_bf16((1, T, Hq, 128), DEV, gen)
    k = synth.randn_bf16((1, Hkv, T, 128), DEV, gen)
    v = synth.randn_bf16((1, Hkv, T, 128), DEV, gen)
    out, lse, gt = seer.attn_ground_truth(q, k, v, b, w.scale)
    torch.cuda.synchronize()
    P = 512
    ro, rl, rg = oracle.attn_ground_truth(q[:, :P].cpu(), k[:, :, :P].cpu(), v[:, :, :P].cpu(), b, w.scale)
    np.testing.assert_allclose(lse[:, :P].cpu().numpy(), rl, rtol=0, atol=1e-3)
    np.testing.assert_allclose(gt[:, :, :P, :P // b].cpu().numpy(), rg, rtol=2e-4, atol=1e-7)
    assert (gt[:, :, :P, P // b:] == 0).all()
    assert np.abs(out[:, :P].float().cpu().numpy() - ro).max() <= 1e-2
    kc, vc = k.cpu(), v.cpu()
    for t in (4095, 8192, 12345, T - 1):
        o1, l1 = oracle.sparse_decode(q[:, t].cpu().contiguous(), oracle.KVLayout(kc, vc),
                                      torch.tensor([t + 1], dtype=torch.int32), None, None, b, w.scale)
        np.testing.assert_allclose(lse[:, t].cpu().numpy(), l1, rtol=0, atol=1e-3)
        assert np.abs(out[:, t].float().cpu().numpy() - o1).max() <= 1e-2
    g = gt.cpu().numpy().astype(np.float64)
    np.testing.assert_allclose(g.sum(-1), 1.0, rtol=0, atol=5e-6)
    rows = np.arange(T)
    visible = (np.arange(T // b)[None, :] <= (rows // b)[:, None])
    assert (g[0][:, ~visible] == 0).all() and (g[0][:, visible] > 0).all()
