"""GPU parity: the HIP library (through the C ABI) against the fp64 CPU oracle, element by
element, on seeded synthetic inputs.  Block indices must match bit-exactly; outputs within the
tolerances in tests/helpers.py.  Sizes are small enough for the oracle to finish in seconds but
span several tiles, several splits and ragged tails.  (The paper prints no worked numeric
example; expectations come from the oracle, which tests/test_oracle_pins.py pins.)"""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2506_08889_amd as seer
import synth
from helpers import check_decode, check_indices, cpu, oracle_decode, oracle_gate, pick_threshold, pick_top_p

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
IMPLS = {"valu": 1, "mfma": 2}


@pytest.fixture(autouse=True)
def _reset_knobs():
    for k in (0, 1, 3):
        seer.set_knob(k, 0)
    yield
    for k in (0, 1, 3):
        seer.set_knob(k, 0)


def gate_both_impls(*args, **kw):
    """seer.gate_select through both gate implementations (score + select kernels, fused kernel);
    the two must agree bit for bit.  Returns the result (the callers compare it with the oracle)."""
    res = []
    for impl in (1, 2):
        seer.set_knob(3, impl)
        idx, cnt = seer.gate_select(*args, **kw)
        torch.cuda.synchronize()
        res.append((idx, cnt))
    seer.set_knob(3, 0)
    for r in res[1:]:
        assert torch.equal(res[0][0], r[0]) and torch.equal(res[0][1], r[1]), "gate implementations differ"
    return res[1]


def gpu_gate(inp, mode=seer.SELECT_TOPK, threshold=0.0, max_sel=None, ragged=False):
    w = inp.w
    return gate_both_impls(inp.q_gate, inp.kc, inp.seqlens, w.block_size, mode=mode,
                           budget_tokens=w.budget_tokens, budget_blocks=inp.budget_blocks,
                           threshold=threshold, max_sel=max_sel or inp.max_sel, ragged=ragged)


def gpu_decode(inp, block_idx, nblk, out_dtype, ragged=False):
    w = inp.w
    return seer.sparse_decode(inp.q, inp.k, inp.v, inp.seqlens, block_idx, nblk, w.block_size, w.scale,
                              page_table=inp.page_table, page_size=inp.page_size, out_dtype=out_dtype, ragged=ragged)


def run_gate_and_decode(w, impls=("valu", "mfma"), splits=(0,), ragged=0):
    print(f"[case] {w.name} B={w.B} Hq={w.Hq} Hkv={w.Hkv} bs={w.block_size} seed={w.seed}", flush=True)
    inp = synth.make_inputs(w, DEV)
    ref_idx, ref_cnt = oracle_gate(inp)
    idx, cnt = gpu_gate(inp, ragged=bool(ragged))
    torch.cuda.synchronize()
    check_indices(idx, cnt, ref_idx, ref_cnt, what=f"{w.name} gate")
    ref_out, ref_lse = oracle_decode(inp, ref_idx, ref_cnt)
    for impl in impls:
        seer.set_knob(0, IMPLS[impl])
        for ns in splits:
            seer.set_knob(1, ns)
            for dt, tight in ((torch.float32, True), (torch.bfloat16, False)):
                print(f"[decode] {w.name} impl={impl} splits={ns} out={dt}", flush=True)
                out, lse = gpu_decode(inp, idx, cnt, dt, ragged=bool(ragged))
                torch.cuda.synchronize()
                check_decode(out, lse, ref_out, ref_lse, tight=tight, what=f"{w.name} {impl} ns={ns} {dt}")
    return inp, idx, cnt, ref_out, ref_lse


# ------------------------------------------------------------ the benchmark configurations, scaled


def test_c1_tiny_single_layer_full_size():
    run_gate_and_decode(synth.CONFIGS["c1"], splits=(0, 1, 3))


def test_c2_shape_scaled():
    w = synth.scaled(synth.CONFIGS["c2"], B=3, seqlen=4096 + 64 * 5, budget_tokens=1024)
    run_gate_and_decode(w, splits=(0, 2))


def test_c3_shape_scaled_paged_varlen_outliers():
    w = synth.scaled(synth.CONFIGS["c3"], B=5, seqlen_range=(900, 6000))
    inp, idx, cnt, _, _ = run_gate_and_decode(w, splits=(0, 5), ragged=1)
    # the ragged tail really is exercised
    assert (inp.seqlens_cpu % w.block_size != 0).any()
    nb = (inp.seqlens_cpu + w.block_size - 1) // w.block_size
    last = cpu(idx).gather(2, (cpu(cnt).long() - 1).clamp(min=0).unsqueeze(-1)).squeeze(-1)
    part = (inp.seqlens_cpu % w.block_size != 0)
    assert (last[part] == (nb[part] - 1).unsqueeze(-1)).all()


def test_c4_shape_scaled_group_of_five():
    w = synth.scaled(synth.CONFIGS["c4"], B=2, seqlen=8192, budget_tokens=819)
    run_gate_and_decode(w, splits=(0, 4))


@pytest.mark.parametrize("bs", [16, 64, 128])
def test_c5_shape_scaled_topk_and_threshold(bs):
    w = synth.scaled(synth.CONFIGS["c5"], B=6, block_size=bs, seqlen_range=(300, 9000), name=f"c5_b{bs}")
    inp, idx, cnt, _, _ = run_gate_and_decode(w, impls=("mfma",), ragged=1)
    # threshold mode at several sparsity levels, thresholds placed between adjacent probabilities
    _, _, scores = oracle_gate(inp, return_scores=True)
    for keep in (0.5, 0.25, 0.10, 0.05):
        tau = pick_threshold(scores, inp.seqlens_cpu, bs, w.Dg, keep)
        ref_idx, ref_cnt = oracle_gate(inp, mode=oracle.SELECT_THRESHOLD, threshold=tau, max_sel=inp.nb_max)
        print(f"[threshold] {w.name} keep={keep} tau={tau:.6g} selected={int(ref_cnt.sum())}", flush=True)
        gi, gc = gpu_gate(inp, mode=seer.SELECT_THRESHOLD, threshold=tau, max_sel=inp.nb_max, ragged=True)
        torch.cuda.synchronize()
        check_indices(gi, gc, ref_idx, ref_cnt, what=f"{w.name} threshold keep={keep}")
        ref_out, ref_lse = oracle_decode(inp, ref_idx, ref_cnt)
        out, lse = gpu_decode(inp, gi, gc, torch.float32, ragged=True)
        torch.cuda.synchronize()
        check_decode(out, lse, ref_out, ref_lse, tight=True, what=f"{w.name} threshold keep={keep}")


# ------------------------------------------------------------------------------- decode edge cases


def small_inputs(seed, B=2, Hq=8, Hkv=2, S=(300, 200), bs=64, paged=False):
    w = synth.Workload("edge", B=B, Hq=Hq, Hkv=Hkv, block_size=bs, seqlen=max(S), paged=paged,
                       budget_tokens=bs * 4, seed=seed)       # cache sized for the longest sequence
    inp = synth.make_inputs(w, "cpu")
    inp.seqlens_cpu = torch.tensor(S, dtype=torch.int32)
    inp.seqlens = inp.seqlens_cpu.clone()
    return inp


def to_dev(inp):
    for f in ("seqlens", "q", "k", "v", "page_table", "q_gate", "kc", "budget_blocks"):
        t = getattr(inp, f)
        if t is not None:
            setattr(inp, f, t.to(DEV))
    return inp


@pytest.mark.parametrize("impl", ["valu", "mfma"])
def test_invalid_entries_permutation_empty_groups(impl):
    seer.set_knob(0, IMPLS[impl])
    inp = to_dev(small_inputs(21, B=3, S=(640, 333, 0)))
    idx = torch.full((3, 2, 8), -1, dtype=torch.int32)
    cnt = torch.zeros(3, 2, dtype=torch.int32)
    idx[0, 0, :6] = torch.tensor([9, 0, -1, 5, 10, 2]); cnt[0, 0] = 6      # unsorted, -1 and 10 (= nb) skipped
    idx[0, 1, :3] = torch.tensor([99, -7, 3]); cnt[0, 1] = 3
    idx[1, 0, :4] = torch.tensor([5, 0, 4, 1]); cnt[1, 0] = 4              # block 5 has 13 tokens
    cnt[1, 1] = 0                                                          # empty selection
    idx[2, :, 0] = 0; cnt[2, :] = 1                                        # empty sequence
    ref_out, ref_lse = oracle_decode(inp, idx, cnt)
    for ns in (0, 1, 2, 8):
        seer.set_knob(1, ns)
        out, lse = gpu_decode(inp, idx.to(DEV), cnt.to(DEV), torch.float32)
        torch.cuda.synchronize()
        check_decode(out, lse, ref_out, ref_lse, tight=True, what=f"edge {impl} ns={ns}")
    # nblk larger than the list capacity is clamped; negative counts mean empty
    cnt2 = cnt.clone(); cnt2[0, 0] = 1000; cnt2[0, 1] = -3
    idx2 = idx.clone()
    ref_out, ref_lse = oracle_decode(inp, idx2, cnt2)
    out, lse = gpu_decode(inp, idx2.to(DEV), cnt2.to(DEV), torch.float32)
    torch.cuda.synchronize()
    check_decode(out, lse, ref_out, ref_lse, tight=True, what=f"edge {impl} clamped counts")


@pytest.mark.parametrize("impl", ["valu", "mfma"])
@pytest.mark.parametrize("g", [1, 2, 3, 4, 5, 6, 7, 8])
def test_every_group_size(impl, g):
    seer.set_knob(0, IMPLS[impl])
    inp = to_dev(small_inputs(30 + g, B=2, Hq=2 * g, Hkv=2, S=(777, 130)))
    gen = torch.Generator().manual_seed(g)
    nb = (inp.seqlens_cpu + 63) // 64
    idx, cnt = synth.random_block_lists(2, 2, nb, [7, 2], 7, gen, ascending=False)
    ref_out, ref_lse = oracle_decode(inp, idx, cnt)
    out, lse = gpu_decode(inp, idx.to(DEV), cnt.to(DEV), torch.float32)
    torch.cuda.synchronize()
    check_decode(out, lse, ref_out, ref_lse, tight=True, what=f"g={g} {impl}")


@pytest.mark.parametrize("bs", [16, 32, 64, 128])
def test_block_sizes_and_dense_decode(bs):
    inp = to_dev(small_inputs(40 + bs, B=2, Hq=8, Hkv=2, S=(1000, 517), bs=bs))
    nbs = (inp.seqlens_cpu + bs - 1) // bs
    gen = torch.Generator().manual_seed(bs)
    k_sel = [max(1, int(n) // 3) for n in nbs]
    idx, cnt = synth.random_block_lists(2, 2, nbs, k_sel, max(k_sel), gen)
    # make sure the partial last block of sequence 0 is in one list
    idx[0, 0, int(cnt[0, 0]) - 1] = int(nbs[0]) - 1
    ref_out, ref_lse = oracle_decode(inp, idx, cnt)
    out, lse = gpu_decode(inp, idx.to(DEV), cnt.to(DEV), torch.float32)
    torch.cuda.synchronize()
    check_decode(out, lse, ref_out, ref_lse, tight=True, what=f"bs={bs} sparse")
    # dense decode == oracle over all blocks
    dref_out, dref_lse = oracle_decode(inp, None, None)
    for impl in ("valu", "mfma"):
        seer.set_knob(0, IMPLS[impl])
        w = inp.w
        out, lse = seer.dense_decode(inp.q, inp.k, inp.v, inp.seqlens, int(nbs.max()), bs, w.scale,
                                     out_dtype=torch.float32)
        torch.cuda.synchronize()
        check_decode(out, lse, dref_out, dref_lse, tight=True, what=f"bs={bs} dense {impl}")


@pytest.mark.parametrize("impl", ["valu", "mfma"])
def test_strided_cache_and_page_size_multiple_of_block(impl):
    seer.set_knob(0, IMPLS[impl])
    inp = to_dev(small_inputs(50, B=2, S=(512, 448)))
    B, Hkv, S_alloc, d = inp.k.shape
    wide_k = torch.zeros(B, Hkv, S_alloc, 2 * d, dtype=torch.bfloat16, device=DEV)
    wide_v = torch.zeros_like(wide_k)
    wide_k[..., :d] = inp.k; wide_v[..., :d] = inp.v
    gen = torch.Generator().manual_seed(5)
    idx, cnt = synth.random_block_lists(2, 2, [8, 7], [5, 4], 5, gen)
    ref_out, ref_lse = oracle_decode(inp, idx, cnt)
    w = inp.w
    out, lse = seer.sparse_decode(inp.q, wide_k[..., :d], wide_v[..., :d], inp.seqlens, idx.to(DEV), cnt.to(DEV),
                                  64, w.scale, out_dtype=torch.float32)
    torch.cuda.synchronize()
    check_decode(out, lse, ref_out, ref_lse, tight=True, what=f"strided {impl}")
    # paged pool whose pages hold two blocks each, pages in reverse order
    npg = S_alloc // 128
    pool_k = torch.zeros(B * npg + 1, Hkv, 128, d, dtype=torch.bfloat16, device=DEV)
    pool_v = torch.zeros_like(pool_k)
    pt = torch.zeros(B, npg, dtype=torch.int32)
    for i in range(B):
        for pg in range(npg):
            phys = B * npg - (i * npg + pg)
            pt[i, pg] = phys
            pool_k[phys] = inp.k[i, :, pg * 128:(pg + 1) * 128]
            pool_v[phys] = inp.v[i, :, pg * 128:(pg + 1) * 128]
    out, lse = seer.sparse_decode(inp.q, pool_k, pool_v, inp.seqlens, idx.to(DEV), cnt.to(DEV), 64, w.scale,
                                  page_table=pt.to(DEV), page_size=128, out_dtype=torch.float32)
    torch.cuda.synchronize()
    check_decode(out, lse, ref_out, ref_lse, tight=True, what=f"paged x2 {impl}")


@pytest.mark.parametrize("impl", ["valu", "mfma"])
def test_needle_and_large_logits(impl):
    """One key aligned with a query gives a logit far above the rest (softmax saturates) and
    a key just past the end of the sequence must never be read."""
    seer.set_knob(0, IMPLS[impl])
    inp = small_inputs(60, B=1, Hq=4, Hkv=1, S=(300,))
    inp.k[0, 0, 299] = (inp.q[0, 1].float() * 6.0).to(torch.bfloat16)      # last valid token of the partial block
    inp.k[0, 0, 300] = (inp.q[0, 1].float() * 60.0).to(torch.bfloat16)     # beyond the sequence
    inp.v[0, 0, 300] = 1000.0
    inp = to_dev(inp)
    idx = torch.tensor([[[1, 4, 3]]], dtype=torch.int32); cnt = torch.tensor([[3]], dtype=torch.int32)
    ref_out, ref_lse = oracle_decode(inp, idx, cnt)
    out, lse = gpu_decode(inp, idx.to(DEV), cnt.to(DEV), torch.float32)
    torch.cuda.synchronize()
    check_decode(out, lse, ref_out, ref_lse, tight=True, what=f"needle {impl}")
    assert abs(float(out[0, 1].float().cpu().numpy() @ np.ones(128)) - float(ref_out[0, 1].sum())) < 0.05


def test_long_list_many_chunks_of_descriptors():
    """A slice longer than 64 list entries (descriptor chunks reload) with one split."""
    seer.set_knob(1, 1)
    inp = to_dev(small_inputs(70, B=1, Hq=8, Hkv=2, S=(64 * 200 + 17,)))
    gen = torch.Generator().manual_seed(70)
    idx, cnt = synth.random_block_lists(1, 2, [201], [150], 150, gen, ascending=False)
    idx[0, 0, 70] = 200          # the partial block somewhere in the middle
    ref_out, ref_lse = oracle_decode(inp, idx, cnt)
    for impl in ("valu", "mfma"):
        seer.set_knob(0, IMPLS[impl])
        out, lse = gpu_decode(inp, idx.to(DEV), cnt.to(DEV), torch.float32)
        torch.cuda.synchronize()
        check_decode(out, lse, ref_out, ref_lse, tight=True, what=f"long list {impl}")


# --------------------------------------------------------------------------------- gate edge cases


def test_gate_ties_and_edge_rules_bit_exact():
    gen = torch.Generator().manual_seed(80)
    B, Hkv, nb_max, bs = 6, 3, 300, 64
    qg = torch.randint(-2, 3, (B, Hkv, 128), generator=gen).to(torch.bfloat16)      # many exact ties
    kc = torch.randint(-1, 2, (B, Hkv, nb_max, 128), generator=gen).to(torch.bfloat16)
    kc[1] = kc[1, 0, 0]                                                             # all scores equal
    sl = torch.tensor([300 * bs, 257 * bs, 256 * bs + 1, 5, 0, 64], dtype=torch.int32)
    for budget in (1, bs, 3 * bs + 1, 100 * bs, 299 * bs, 10 ** 6):
        max_sel = min((budget + bs - 1) // bs, nb_max)
        ri, rc = oracle.gate_select(qg, kc, sl, bs, budget_tokens=budget, max_sel=max_sel)
        gi, gc = gate_both_impls(qg.to(DEV), kc.to(DEV), sl.to(DEV), bs, budget_tokens=budget, max_sel=max_sel)
        torch.cuda.synchronize()
        check_indices(gi, gc, ri, rc, what=f"ties budget={budget}")
    # per-sequence block budgets, including 0 and more than there are blocks; wider list than needed
    bb = torch.tensor([7, 0, 400, 3, 2, 1], dtype=torch.int32)
    ri, rc = oracle.gate_select(qg, kc, sl, bs, budget_blocks=bb, max_sel=310)
    gi, gc = gate_both_impls(qg.to(DEV), kc.to(DEV), sl.to(DEV), bs, budget_blocks=bb.to(DEV), max_sel=310)
    torch.cuda.synchronize()
    check_indices(gi, gc, ri, rc, what="budget_blocks")
    # list narrower than a per-sequence budget: clamped to max_sel
    ri, rc = oracle.gate_select(qg, kc, sl, bs, budget_blocks=bb, max_sel=5)
    gi, gc = gate_both_impls(qg.to(DEV), kc.to(DEV), sl.to(DEV), bs, budget_blocks=bb.to(DEV), max_sel=5)
    torch.cuda.synchronize()
    check_indices(gi, gc, ri, rc, what="budget_blocks clamped")
    # threshold: strict comparison on exactly representable probabilities (4 equal scores -> 1/4)
    kc4 = kc[:, :, :4].clone(); kc4[:] = kc[0, 0, 0]
    sl4 = torch.full((B,), 4 * bs, dtype=torch.int32)
    for tau in (0.25, 0.2499999, 0.0, 1.0):
        ri, rc = oracle.gate_select(qg, kc4, sl4, bs, mode=oracle.SELECT_THRESHOLD, threshold=tau, max_sel=4)
        gi, gc = gate_both_impls(qg.to(DEV), kc4.to(DEV), sl4.to(DEV), bs, mode=seer.SELECT_THRESHOLD,
                                  threshold=tau, max_sel=4)
        torch.cuda.synchronize()
        check_indices(gi, gc, ri, rc, what=f"threshold tau={tau}")


def test_gate_strided_compression_cache_and_long_context():
    gen = torch.Generator().manual_seed(81)
    B, Hkv, nb_max, bs = 2, 8, 2048, 64
    qg = torch.randn(B, Hkv, 128, generator=gen).to(torch.bfloat16)
    wide = torch.randn(B, Hkv, nb_max, 256, generator=gen).to(torch.bfloat16)
    kc = wide[..., 128:]                                         # row stride 256, offset 128
    sl = torch.tensor([131072, 131072 - 63], dtype=torch.int32)
    ri, rc = oracle.gate_select(qg, kc, sl, bs, budget_tokens=13107, max_sel=205)
    wd = wide.to(DEV)
    gi, gc = gate_both_impls(qg.to(DEV), wd[..., 128:], sl.to(DEV), bs, budget_tokens=13107, max_sel=205)
    torch.cuda.synchronize()
    check_indices(gi, gc, ri, rc, what="strided kc, 2048 blocks")


def test_results_are_deterministic_run_to_run():
    w = synth.scaled(synth.CONFIGS["c2"], B=2, seqlen=2048, budget_tokens=512)
    inp = synth.make_inputs(w, DEV)
    idx, cnt = gpu_gate(inp)
    a = gpu_decode(inp, idx, cnt, torch.float32)
    b = gpu_decode(inp, idx, cnt, torch.float32)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    idx2, cnt2 = gpu_gate(inp)
    torch.cuda.synchronize()
    assert torch.equal(idx, idx2) and torch.equal(cnt, cnt2)


def test_hip_graph_capture_and_replay_match_eager():
    """The two calls allocate nothing, never synchronise and record no memset, so a step can be
    captured into a HIP graph; every replay must reproduce the eager result bit for bit, with eager
    work and synchronisations between the replays."""
    w = synth.scaled(synth.CONFIGS["c2"], B=2, seqlen=4096, budget_tokens=1024)
    inp = synth.make_inputs(w, DEV)
    B, Hq, Hkv, d = w.B, w.Hq, w.Hkv, w.d
    idx = torch.empty(B, Hkv, inp.max_sel, dtype=torch.int32, device=DEV)
    cnt = torch.empty(B, Hkv, dtype=torch.int32, device=DEV)
    out = torch.empty(B, Hq, d, dtype=torch.float32, device=DEV)
    lse = torch.empty(B, Hq, dtype=torch.float32, device=DEV)
    wsg = torch.empty(seer.gate_workspace_bytes(B, Hkv, inp.nb_max), dtype=torch.uint8, device=DEV)
    wsd = torch.empty(seer.decode_workspace_bytes(B, Hq, Hkv, d, inp.max_sel), dtype=torch.uint8, device=DEV)
    seer.set_knob(1, 4)      # several splits: split kernel + merge kernel are both in the graph

    def step():
        seer.gate_select(inp.q_gate, inp.kc, inp.seqlens, w.block_size, budget_tokens=w.budget_tokens,
                         max_sel=inp.max_sel, block_idx=idx, nblk=cnt, workspace=wsg)
        seer.sparse_decode(inp.q, inp.k, inp.v, inp.seqlens, idx, cnt, w.block_size, w.scale, out=out, lse=lse,
                           workspace=wsd)

    step()
    torch.cuda.synchronize()
    ref = (idx.clone(), cnt.clone(), out.clone(), lse.clone())
    s = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(s):
        with torch.cuda.graph(g, stream=s):
            step()
    torch.cuda.synchronize()
    for rep in range(4):
        for t in (idx, cnt, out, lse):
            t.zero_()
        (inp.q.float() * 2).sum().item()          # unrelated eager work + a synchronisation
        g.replay()
        torch.cuda.synchronize()
        for got, want in zip((idx, cnt, out, lse), ref):
            assert torch.equal(got, want), f"replay {rep} differs from the eager result"


@pytest.mark.parametrize("impl", ["valu", "mfma"])
@pytest.mark.parametrize("ns", [1, 3, 5])
def test_needles_at_slice_and_block_boundaries(impl, ns):
    """A key aligned with one query head (logit far above the rest) placed, in turn, at the first
    token of the first listed block, the first and last token of the first and last block of every
    slice of the list, the last valid token of the partial block, and in an unselected block (must
    change nothing).  Catches gather-addressing, tail-masking and slice-boundary mistakes that the
    1e-2 tolerance would hide on plain random data."""
    seer.set_knob(0, IMPLS[impl])
    seer.set_knob(1, ns)
    bs, nsel = 64, 23
    base = small_inputs(90 + ns, B=1, Hq=8, Hkv=2, S=(64 * 40 + 21,))
    gen = torch.Generator().manual_seed(7)
    idx, cnt = synth.random_block_lists(1, 2, [41], [nsel], nsel, gen, ascending=False)
    idx[0, 0, 11] = 40                                    # the partial block (21 tokens) inside the list
    idx[0, 1] = idx[0, 0]
    listed = idx[0, 0].tolist()
    assert len(set(listed)) == nsel
    unselected = next(j for j in range(40) if j not in listed)
    L = -(-nsel // ns)
    spots = [(listed[0], 0)]
    for s in range(0, nsel, L):
        first, last = listed[s], listed[min(s + L, nsel) - 1]
        for blk in (first, last):
            ntok = 21 if blk == 40 else bs
            spots += [(blk, 0), (blk, ntok - 1)]
    spots += [(40, 20), (unselected, 5)]
    dev_idx, dev_cnt = idx.to(DEV), cnt.to(DEV)
    for blk, tok in dict.fromkeys(spots):
        inp = small_inputs(90 + ns, B=1, Hq=8, Hkv=2, S=(64 * 40 + 21,))
        pos = blk * bs + tok
        inp.k[0, 0, pos] = (inp.q[0, 2].float() * 5.0).to(torch.bfloat16)     # head 2 -> kv head 0
        inp.k[0, 1, pos] = (inp.q[0, 5].float() * 5.0).to(torch.bfloat16)     # head 5 -> kv head 1
        inp = to_dev(inp)
        ref_out, ref_lse = oracle_decode(inp, idx, cnt)
        out, lse = gpu_decode(inp, dev_idx, dev_cnt, torch.float32)
        torch.cuda.synchronize()
        check_decode(out, lse, ref_out, ref_lse, tight=True, what=f"needle at block {blk} token {tok} ({impl}, ns={ns})")
        if blk != unselected:      # the needle really dominates its head
            v_row = inp.v[0, 0, pos].float().cpu().numpy()
            assert np.abs(ref_out[0, 2] - v_row).max() < 0.05


@pytest.mark.parametrize("bs", [64, 128])
def test_top_p_selection_and_decode(bs):
    """Nucleus (top-p) block selection, bit-exact against the oracle, then decode on the ragged lists."""
    w = synth.scaled(synth.CONFIGS["c5"], B=6, block_size=bs, seqlen_range=(300, 9000), name=f"topp_b{bs}")
    inp = synth.make_inputs(w, DEV)
    _, _, scores = oracle_gate(inp, return_scores=True)
    for lo, hi in ((0.2, 0.4), (0.5, 0.7), (0.85, 0.97)):
        p = pick_top_p(scores, inp.seqlens_cpu, bs, w.Dg, lo, hi)
        ref_idx, ref_cnt = oracle_gate(inp, mode=oracle.SELECT_TOPP, threshold=p, max_sel=inp.nb_max)
        print(f"[top-p] {w.name} p={p:.6f} selected={int(ref_cnt.sum())}", flush=True)
        gi, gc = gpu_gate(inp, mode=seer.SELECT_TOPP, threshold=p, max_sel=inp.nb_max, ragged=True)
        check_indices(gi, gc, ref_idx, ref_cnt, what=f"{w.name} top-p {p:.4f}")
        ref_out, ref_lse = oracle_decode(inp, ref_idx, ref_cnt)
        out, lse = gpu_decode(inp, gi, gc, torch.float32, ragged=True)
        torch.cuda.synchronize()
        check_decode(out, lse, ref_out, ref_lse, tight=True, what=f"{w.name} top-p {p:.4f}")
    # edge values of p and exact ties
    # edge values of p (p >= 1 is the whole mass: every full block, on both sides) and exact ties
    nfull = (inp.seqlens_cpu // bs).numpy()
    nbs = ((inp.seqlens_cpu + bs - 1) // bs).numpy()
    for p in (0.0, 1.0, 7.0, -1.0):
        ref_idx, ref_cnt = oracle_gate(inp, mode=oracle.SELECT_TOPP, threshold=p, max_sel=inp.nb_max)
        gi, gc = gpu_gate(inp, mode=seer.SELECT_TOPP, threshold=p, max_sel=inp.nb_max)
        check_indices(gi, gc, ref_idx, ref_cnt, what=f"top-p edge p={p}")
        if p >= 1.0:
            assert (ref_cnt == np.minimum(nbs, inp.nb_max)[:, None]).all()
        if p <= 0.0:
            assert (ref_cnt == (np.minimum(nfull, 1) + (nbs > nfull))[:, None]).all()
    gen = torch.Generator().manual_seed(3)
    qg = torch.randint(-2, 3, (2, 2, 128), generator=gen).to(torch.bfloat16)
    kc = torch.randint(-1, 2, (2, 2, 40, 128), generator=gen).to(torch.bfloat16)
    kc[1] = kc[1, 0, 0]                                   # 40 equal scores: probability 1/40 each
    sl = torch.tensor([40 * bs, 40 * bs], dtype=torch.int32)
    for p in (0.26, 0.5001, 0.999):
        ri, rc = oracle.gate_select(qg, kc, sl, bs, mode=oracle.SELECT_TOPP, threshold=p, max_sel=40)
        gi, gc = gate_both_impls(qg.to(DEV), kc.to(DEV), sl.to(DEV), bs, mode=seer.SELECT_TOPP, threshold=p, max_sel=40)
        check_indices(gi[1:], gc[1:], ri[1:], rc[1:], what=f"top-p ties p={p}")


def test_randomised_shapes_gate_and_decode():
    """Forty seeded random configurations (group size, block size, batch, lengths incl. empty and
    sub-block sequences, contiguous/paged, selection mode, split plan): indices bit-exact, outputs
    within the tight fp32-output bars."""
    rng = np.random.default_rng(2024)
    for case in range(40):
        g = int(rng.integers(1, 9))
        Hkv = int(rng.choice([1, 2, 3, 8]))
        bs = int(rng.choice([16, 32, 64, 128]))
        B = int(rng.integers(1, 6))
        paged = bool(rng.integers(0, 2))
        hi = int(rng.choice([bs * 3, bs * 20, bs * 70]))
        w = synth.Workload(f"rand{case}", B=B, Hq=g * Hkv, Hkv=Hkv, block_size=bs, seqlen_range=(1, hi),
                           seqlen_dist="uniform", paged=paged, budget_tokens=0, budget_frac=float(rng.choice([0.1, 0.3, 1.0])),
                           seed=1000 + case)
        inp = synth.make_inputs(w, DEV)
        # some sequences empty or shorter than a block
        sl = inp.seqlens_cpu.clone()
        if B > 1 and case % 3 == 0:
            sl[0] = int(rng.choice([0, 1, bs - 1, bs]))
        inp.seqlens_cpu = sl
        inp.seqlens = sl.to(DEV)
        mode = [seer.SELECT_TOPK, seer.SELECT_THRESHOLD, seer.SELECT_TOPP][case % 3]
        max_sel = inp.nb_max if mode != seer.SELECT_TOPK else inp.max_sel
        thr = 0.0
        if mode != seer.SELECT_TOPK:
            _, _, scores = oracle_gate(inp, return_scores=True)
            if (sl // bs).max() == 0:
                mode, max_sel = seer.SELECT_TOPK, inp.max_sel
            elif mode == seer.SELECT_THRESHOLD:
                thr = pick_threshold(scores, sl, bs, w.Dg, float(rng.choice([0.5, 0.2])))
            else:
                thr = pick_top_p(scores, sl, bs, w.Dg, 0.3, 0.9, seed=case)
        print(f"[rand {case}] g={g} Hkv={Hkv} bs={bs} B={B} paged={paged} mode={mode} seqlens={sl.tolist()}", flush=True)
        ref_idx, ref_cnt = oracle_gate(inp, mode=mode, threshold=thr, max_sel=max_sel)
        gi, gc = gpu_gate(inp, mode=mode, threshold=thr, max_sel=max_sel, ragged=bool(case & 1))
        check_indices(gi, gc, ref_idx, ref_cnt, what=f"rand {case} gate")
        ref_out, ref_lse = oracle_decode(inp, ref_idx, ref_cnt)
        seer.set_knob(1, int(rng.choice([0, 1, 2, 7])))
        out, lse = gpu_decode(inp, gi, gc, torch.float32, ragged=bool(rng.integers(0, 2)))
        torch.cuda.synchronize()
        check_decode(out, lse, ref_out, ref_lse, tight=True, what=f"rand {case} decode")
        seer.set_knob(1, 0)
        dref_out, dref_lse = oracle_decode(inp, None, None)
        out, lse = seer.dense_decode(inp.q, inp.k, inp.v, inp.seqlens, inp.nb_max, bs, w.scale,
                                     page_table=inp.page_table, page_size=inp.page_size, out_dtype=torch.float32)
        torch.cuda.synchronize()
        check_decode(out, lse, dref_out, dref_lse, tight=True, what=f"rand {case} dense")


@pytest.mark.parametrize("g,T,bs", [(4, 4, 64), (5, 3, 64), (2, 8, 128), (8, 2, 32), (4, 1, 64), (1, 16, 64), (4, 3, 16)])
def test_multi_token_decode(g, T, bs):
    """q_len new tokens per sequence in one call: each query against the oracle (causal among the
    new tokens, shared block list), for several split plans; sequences shorter than q_len included."""
    Hkv = 2
    S = (bs * 9 + 5, bs * 4, T - 1 if T > 1 else 1, bs * 6 + bs // 2 + 1)
    w = synth.Workload("mtp", B=4, Hq=g * Hkv, Hkv=Hkv, block_size=bs, seqlen=max(S), budget_tokens=bs * 4, seed=500 + g * T)
    inp = synth.make_inputs(w, "cpu")
    inp.seqlens_cpu = torch.tensor(S, dtype=torch.int32)
    inp.seqlens = inp.seqlens_cpu.clone()
    inp = to_dev(inp)
    gen = torch.Generator().manual_seed(g * 100 + T)
    qm = torch.randn(4, T, g * Hkv, 128, generator=gen).to(torch.bfloat16)
    nb = (inp.seqlens_cpu + bs - 1) // bs
    idx, cnt = synth.random_block_lists(4, Hkv, nb, [6, 3, 1, 5], 6, gen, ascending=False)
    for i in range(4):           # the last block (where the causal limits bite) is always listed
        if int(nb[i]) > 0 and (idx[i, 0, :int(cnt[i, 0])] == int(nb[i]) - 1).sum() == 0:
            idx[i, :, 0] = int(nb[i]) - 1
    ref_out, ref_lse = oracle.sparse_decode_multi(qm, oracle.KVLayout(cpu(inp.k), cpu(inp.v)), inp.seqlens_cpu, idx, cnt,
                                                  bs, w.scale)
    for ns in (0, 1, 3):
        seer.set_knob(1, ns)
        out, lse = seer.sparse_decode_multi(qm.to(DEV), inp.k, inp.v, inp.seqlens, idx.to(DEV), cnt.to(DEV), bs, w.scale,
                                            out_dtype=torch.float32)
        torch.cuda.synchronize()
        check_decode(out.view(4, T * g * Hkv, 128), lse.view(4, T * g * Hkv), ref_out.reshape(4, T * g * Hkv, 128),
                     ref_lse.reshape(4, T * g * Hkv), tight=True, what=f"multi-token g={g} T={T} bs={bs} ns={ns}")
    if T == 1:                   # one new token is the plain call
        o1, l1 = gpu_decode(inp, idx.to(DEV), cnt.to(DEV), torch.float32)
        o1 = o1.clone(); inp.q = qm[:, 0].contiguous().to(DEV)
        o2, l2 = gpu_decode(inp, idx.to(DEV), cnt.to(DEV), torch.float32)
        assert torch.equal(o2, out[:, 0]) and torch.equal(l2, lse[:, 0])
    # too many rows for the tile / unsupported block size are refused, not mis-computed
    if g * T == 16:
        with pytest.raises(seer.SeerError):
            seer.sparse_decode_multi(torch.zeros(4, T + 1, g * Hkv, 128, dtype=torch.bfloat16, device=DEV), inp.k, inp.v,
                                     inp.seqlens, idx.to(DEV), cnt.to(DEV), bs, w.scale)


def test_pure_c_program_through_the_abi():
    """tests/c_abi/c_abi_check.c uses the library from plain C (HIP runtime allocations, no torch)
    and compares with the C oracle itself; built by __graft_entry__.build()."""
    import os
    import subprocess
    exe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_abi", "c_abi_check")
    if not os.path.exists(exe):
        import __graft_entry__
        __graft_entry__.build_c_abi_check()
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    print(r.stdout, r.stderr)
    assert r.returncode == 0, f"c_abi_check failed with {r.returncode}: {r.stderr}"
    assert "indices bit-exact" in r.stdout


def test_gate_very_long_cache_and_crowded_boundary():
    """(a) A compression cache longer than the select kernel keeps in LDS (> 8192 blocks): scores are
    re-read from global memory and only the radix walk is available.  (b) A boundary bin holding more
    equal scores than the fast path ranks exactly: it must fall back, ties still lowest index first."""
    gen = torch.Generator().manual_seed(91)
    B, Hkv, nb_max, bs = 1, 2, 8300, 16
    qg = torch.randn(B, Hkv, 128, generator=gen).to(torch.bfloat16)
    kc = torch.randn(B, Hkv, nb_max, 128, generator=gen).to(torch.bfloat16)
    sl = torch.tensor([nb_max * bs - 3], dtype=torch.int32)          # last block partial
    for mode, kw in ((seer.SELECT_TOPK, dict(budget_tokens=700 * bs, max_sel=700)),
                     (seer.SELECT_THRESHOLD, dict(threshold=2.0e-4, max_sel=nb_max)),
                     (seer.SELECT_TOPP, dict(threshold=0.6, max_sel=nb_max))):
        ri, rc = oracle.gate_select(qg, kc, sl, bs, mode=mode, **kw)
        gi, gc = seer.gate_select(qg.to(DEV), kc.to(DEV), sl.to(DEV), bs, mode=mode, **kw)
        torch.cuda.synchronize()
        check_indices(gi, gc, ri, rc, what=f"8300-block cache mode={mode}")
    # (a') 20 000 blocks of small-integer data (many equal scores): the ordered compaction runs three passes of
    # 8192 blocks and the radix walk settles ties that straddle the passes
    nb3 = 20000
    gnp = np.random.default_rng(92)
    qg3 = torch.from_numpy(gnp.integers(-2, 3, size=(1, 2, 128)).astype(np.float32)).to(torch.bfloat16)
    kc3 = torch.from_numpy(gnp.integers(-1, 2, size=(1, 2, nb3, 128)).astype(np.float32)).to(torch.bfloat16)
    sl3 = torch.tensor([nb3 * bs - 5], dtype=torch.int32)
    for k in (1, 6000, 19999):
        ri, rc = oracle.gate_select(qg3, kc3, sl3, bs, budget_tokens=k * bs, max_sel=k)
        gi, gc = seer.gate_select(qg3.to(DEV), kc3.to(DEV), sl3.to(DEV), bs, budget_tokens=k * bs, max_sel=k)
        torch.cuda.synchronize()
        check_indices(gi, gc, ri, rc, what=f"20000-block cache k={k}")
    # (b) 900 of 1000 blocks share one score, the k-th largest falls among them
    nb2 = 1000
    kc2 = torch.randn(1, 2, nb2, 128, generator=gen).to(torch.bfloat16)
    same = torch.randperm(nb2, generator=gen)[:900]
    kc2[0, :, same] = kc2[0, :, same[0]].unsqueeze(1)
    sl2 = torch.tensor([nb2 * 64], dtype=torch.int32)
    for budget_blocks in (30, 400, 950):
        ri, rc = oracle.gate_select(qg, kc2, sl2, 64, budget_tokens=budget_blocks * 64, max_sel=budget_blocks)
        gi, gc = gate_both_impls(qg.to(DEV), kc2.to(DEV), sl2.to(DEV), 64, budget_tokens=budget_blocks * 64,
                                 max_sel=budget_blocks)
        check_indices(gi, gc, ri, rc, what=f"crowded boundary k={budget_blocks}")


@pytest.mark.parametrize("seed", [11, 12])
def test_gate_random_shapes_with_many_equal_scores(seed):
    """Token-budget selection on 60 random shapes per seed: batch 1-4, 1-3 kv heads, every block size, caches
    from 1 to 3000 blocks (and the sizes around the kernel's 256 / 512 / 1024 / 8192 steps), sequence
    lengths from empty to full, global and per-sequence budgets from nothing to everything; inputs of small
    integers, constant rows or a handful of distinct rows, so that equal scores are the rule and the
    lowest-index rule decides most lists.  Both gate forms, bit-exact against the oracle."""
    rng = np.random.default_rng(seed)
    for case in range(60):
        B, Hkv, bs = int(rng.integers(1, 5)), int(rng.integers(1, 4)), int(rng.choice([16, 32, 64, 128]))
        nb_max = int(rng.choice([1, 2, 3, 5, 17, 64, 100, 255, 256, 257, 511, 512, 513, 700, 1024, 1500, 2048, 2500, 3000, 8192, 8200]))
        if rng.random() < 0.3:
            nb_max = int(rng.integers(1, 3001))
        seqlens = rng.integers(0, nb_max * bs + 1, size=B).astype(np.int32)
        seqlens[rng.integers(0, B)] = nb_max * bs - int(rng.integers(0, bs))      # one nearly full sequence
        kind = rng.choice(["ties", "normal", "const", "few"])
        if kind == "ties":
            q = rng.integers(-2, 3, size=(B, Hkv, 128)).astype(np.float32)
            kc = rng.integers(-1, 2, size=(B, Hkv, nb_max, 128)).astype(np.float32)
        elif kind == "const":
            q, kc = np.ones((B, Hkv, 128), np.float32), np.ones((B, Hkv, nb_max, 128), np.float32)
        elif kind == "few":
            q = rng.standard_normal((B, Hkv, 128)).astype(np.float32)
            kc = rng.standard_normal((4, 128)).astype(np.float32)[rng.integers(0, 4, size=(B, Hkv, nb_max))]
        else:
            q = rng.standard_normal((B, Hkv, 128)).astype(np.float32)
            kc = rng.standard_normal((B, Hkv, nb_max, 128)).astype(np.float32)
        qg, kct, sl = torch.from_numpy(q).to(torch.bfloat16), torch.from_numpy(kc).to(torch.bfloat16), torch.from_numpy(seqlens)
        if rng.random() < 0.5:
            bb, bt = None, int(rng.integers(0, nb_max * bs + 1))
            k = min(-(-bt // bs), nb_max)
        else:
            bbn = rng.integers(0, nb_max + 2, size=B).astype(np.int32)
            bb, bt, k = torch.from_numpy(bbn), 0, int(min(bbn.max(), nb_max))
        max_sel = max(1, k)
        ri, rc = oracle.gate_select(qg, kct, sl, bs, budget_tokens=bt, budget_blocks=bb, max_sel=max_sel)
        gi, gc = gate_both_impls(qg.to(DEV), kct.to(DEV), sl.to(DEV), bs, budget_tokens=bt,
                                 budget_blocks=None if bb is None else bb.to(DEV), max_sel=max_sel,
                                 ragged=bool(rng.random() < 0.5))
        check_indices(gi, gc, ri, rc, what=f"seed {seed} case {case}: {kind} B={B} Hkv={Hkv} bs={bs} nb_max={nb_max} "
                                            f"budget_tokens={bt} budget_blocks={None if bb is None else bb.tolist()} "
                                            f"seqlens={seqlens.tolist()}")


@pytest.mark.parametrize("nb_max", [6144, 8192])
def test_gate_cache_lengths_whose_scores_need_more_than_64k_of_lds(nb_max):
    """6144 and 8192 blocks (16-token blocks on 96 k / 128 k tokens): the select kernel's LDS copy of the
    scores (9 bytes per block on top of its static arrays) passes 64 KiB; the launch must either get that
    much LDS or fall back to scores in global memory - all three modes, both gate implementations,
    bit-exact either way.  One sequence ends on a partial block, one is far shorter than the cache."""
    gen = torch.Generator().manual_seed(nb_max)
    B, Hkv, bs = 2, 2, 16
    qg = torch.randn(B, Hkv, 128, generator=gen).to(torch.bfloat16)
    kc = torch.randn(B, Hkv, nb_max, 128, generator=gen).to(torch.bfloat16)
    sl = torch.tensor([nb_max * bs - 5, 1500 * bs], dtype=torch.int32)
    _, _, scores = oracle.gate_select(qg, kc, sl, bs, budget_tokens=bs, max_sel=1, return_scores=True)
    tau = pick_threshold(scores, sl, bs, 128, 0.08)
    p = pick_top_p(scores, sl, bs, 128, 0.5, 0.8)
    qd, kd, sd = qg.to(DEV), kc.to(DEV), sl.to(DEV)
    for mode, kw in ((seer.SELECT_TOPK, dict(budget_tokens=600 * bs, max_sel=600)),
                     (seer.SELECT_TOPK, dict(budget_tokens=(nb_max - 7) * bs, max_sel=nb_max)),
                     (seer.SELECT_THRESHOLD, dict(threshold=tau, max_sel=nb_max)),
                     (seer.SELECT_TOPP, dict(threshold=p, max_sel=nb_max))):
        print(f"[lds] nb_max={nb_max} mode={mode} {kw}", flush=True)
        ri, rc = oracle.gate_select(qg, kc, sl, bs, mode=mode, **kw)
        gi, gc = gate_both_impls(qd, kd, sd, bs, mode=mode, **kw)
        check_indices(gi, gc, ri, rc, what=f"nb_max={nb_max} mode={mode}")


def test_multi_token_decode_on_a_paged_cache():
    """q_len new tokens per call on a paged pool: pages of one block and of two blocks, shuffled page
    table, the last block partial (where the causal limits among the new tokens bite)."""
    g, T, Hkv, bs, B = 4, 3, 2, 64, 3
    for page_blocks in (1, 2):
        w = synth.Workload("mtp_paged", B=B, Hq=g * Hkv, Hkv=Hkv, block_size=bs, seqlen_range=(bs * 5, bs * 23 + 31),
                           seqlen_dist="uniform", paged=True, budget_tokens=bs * 4, seed=640 + page_blocks)
        inp = synth.make_inputs(w, DEV)                       # pool with pages of one block
        S = inp.seqlens_cpu.clone(); S[0] = bs * 11 + 2       # two tokens into the last block
        inp.seqlens_cpu = S; inp.seqlens = S.to(DEV)
        k, v, pt, page = inp.k, inp.v, inp.page_table, bs
        if page_blocks == 2:                                  # the same tokens in pages of two blocks
            page = 2 * bs
            ptc = inp.page_table.cpu()
            npg = (inp.nb_max + 1) // 2
            pool_k = torch.zeros(B * npg + 1, Hkv, page, 128, dtype=torch.bfloat16, device=DEV)
            pool_v = torch.zeros_like(pool_k)
            pt2 = torch.zeros(B, npg, dtype=torch.int32)
            order = torch.randperm(B * npg, generator=torch.Generator().manual_seed(9)) + 1
            for i in range(B):
                for pg in range(npg):
                    phys = int(order[i * npg + pg]); pt2[i, pg] = phys
                    for half in range(2):
                        j = 2 * pg + half
                        if j < inp.nb_max and int(ptc[i, j]) > 0:
                            pool_k[phys, :, half * bs:(half + 1) * bs] = inp.k[int(ptc[i, j])]
                            pool_v[phys, :, half * bs:(half + 1) * bs] = inp.v[int(ptc[i, j])]
            k, v, pt = pool_k, pool_v, pt2.to(DEV)
        gen = torch.Generator().manual_seed(77 + page_blocks)
        qm = torch.randn(B, T, g * Hkv, 128, generator=gen).to(torch.bfloat16)
        nb = (S + bs - 1) // bs
        idx = torch.full((B, Hkv, 6), -1, dtype=torch.int32)
        cnt = torch.zeros(B, Hkv, dtype=torch.int32)
        for i in range(B):                                    # the last block (first in the list) + random others
            for h in range(Hkv):
                k_sel = [6, 4, 5][i]
                others = torch.randperm(int(nb[i]) - 1, generator=gen)[:k_sel - 1].tolist()
                idx[i, h, :k_sel] = torch.tensor([int(nb[i]) - 1] + others, dtype=torch.int32)
                cnt[i, h] = k_sel
        ref_out, ref_lse = oracle.sparse_decode_multi(qm, oracle.KVLayout(cpu(k), cpu(v), cpu(pt), page), S, idx, cnt,
                                                      bs, w.scale)
        for ns in (0, 1, 3):
            seer.set_knob(1, ns)
            out, lse = seer.sparse_decode_multi(qm.to(DEV), k, v, inp.seqlens, idx.to(DEV), cnt.to(DEV), bs, w.scale,
                                                page_table=pt, page_size=page, out_dtype=torch.float32)
            torch.cuda.synchronize()
            check_decode(out.view(B, T * g * Hkv, 128), lse.view(B, T * g * Hkv), ref_out.reshape(B, T * g * Hkv, 128),
                         ref_lse.reshape(B, T * g * Hkv), tight=True, what=f"paged multi-token page={page} ns={ns}")
        seer.set_knob(1, 0)


@pytest.mark.parametrize("B,Hkv,smax", [(7, 2, 64 * 400), (80, 8, 64 * 90), (300, 8, 64 * 40)])
def test_ragged_lists_hint_hand_out_of_slices(B, Hkv, smax):
    """With the ragged-lists hint a fixed set of work-groups walks the slices that exist: fewer groups than
    work-groups, more groups than work-groups (the first slices of the later groups are handed out too) and
    more groups than the unit table holds (falls back to one work-group per slice).  A workspace full of
    arbitrary bytes (hand-out word invalid: round-robin), the same workspace again (word left valid by
    the merge: handed out by the counter) and a zeroed one must give bit-identical results; threshold-like
    lists from empty to nearly everything; dense decode on the same mixed lengths."""
    g, bs = 2, 64
    w = synth.Workload("ragged", B=B, Hq=g * Hkv, Hkv=Hkv, block_size=bs, seqlen_range=(1, smax), seqlen_dist="loguniform",
                       paged=True, budget_tokens=0, budget_frac=0.5, seed=B)
    inp = synth.make_inputs(w, DEV)
    nb = (inp.seqlens_cpu + bs - 1) // bs
    rng = np.random.default_rng(B)
    k_sel = [int(rng.integers(0, int(n) + 1)) for n in nb]             # 0 .. all blocks of the sequence
    idx, cnt = synth.random_block_lists(B, Hkv, nb, k_sel, inp.nb_max, torch.Generator().manual_seed(B), ascending=False)
    cnt[0, 0] = 0                                                      # an empty list among non-empty ones
    ref_out, ref_lse = oracle_decode(inp, idx, cnt)
    d_idx, d_cnt = idx.to(DEV), cnt.to(DEV)
    nbytes = seer.decode_workspace_bytes(B, w.Hq, Hkv, w.d, inp.nb_max)
    ws = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device=DEV)
    outs = []
    for label, wsp in (("arbitrary bytes", ws), ("same workspace again", ws), ("zeros", torch.zeros_like(ws))):
        out, lse = seer.sparse_decode(inp.q, inp.k, inp.v, inp.seqlens, d_idx, d_cnt, bs, w.scale, page_table=inp.page_table,
                                      page_size=inp.page_size, out_dtype=torch.float32, workspace=wsp, ragged=True)
        torch.cuda.synchronize()
        check_decode(out, lse, ref_out, ref_lse, tight=True, what=f"ragged B={B} ({label})")
        outs.append((out.clone(), lse.clone()))
    for o, l in outs[1:]:
        assert torch.equal(o, outs[0][0]) and torch.equal(l, outs[0][1]), "the hand-out order changed a result"
    dref_out, dref_lse = oracle_decode(inp, None, None)
    out, lse = seer.dense_decode(inp.q, inp.k, inp.v, inp.seqlens, inp.nb_max, bs, w.scale, page_table=inp.page_table,
                                 page_size=inp.page_size, out_dtype=torch.float32, ragged=True)
    torch.cuda.synchronize()
    check_decode(out, lse, dref_out, dref_lse, tight=True, what=f"ragged dense B={B}")


def test_ragged_lists_hint_on_random_shapes():
    """The slice hand-out on 16 random shapes: 1-8 kv heads, groups of 1-8 heads, every block size, batches
    from 1 to 300 sequences of log-uniform lengths (paged or not), lists from empty to everything in random
    order, a workspace of arbitrary bytes; fp32 output at the tight bars, and a second call on the same
    workspace (hand-out word now valid) must reproduce the first bit for bit."""
    rng = np.random.default_rng(2024)
    for case in range(16):
        Hkv, g, bs = int(rng.choice([1, 2, 3, 8])), int(rng.integers(1, 9)), int(rng.choice([16, 32, 64, 128]))
        B = int(rng.choice([1, 2, 5, 17, 40, 70, 300])) if Hkv < 8 else int(rng.choice([1, 3, 20, 64, 257]))
        smax = int(rng.choice([bs * 40, bs * 150, 2048 * 6 + 5, 2048 * 20 + 77]))
        smax = max(2, min(smax, 200000 // max(1, B // 8)))
        w = synth.Workload("rr", B=B, Hq=g * Hkv, Hkv=Hkv, block_size=bs, seqlen_range=(1, smax), seqlen_dist="loguniform",
                           paged=bool(rng.random() < 0.5), budget_tokens=0, budget_frac=0.5, seed=int(rng.integers(1, 1 << 30)))
        inp = synth.make_inputs(w, DEV)
        nb = (inp.seqlens_cpu + bs - 1) // bs
        k_sel = [int(rng.integers(0, int(n) + 1)) for n in nb]
        idx, cnt = synth.random_block_lists(B, Hkv, nb, k_sel, inp.nb_max, torch.Generator().manual_seed(case),
                                            ascending=bool(rng.random() < 0.5))
        ref_out, ref_lse = oracle_decode(inp, idx, cnt)
        ws = torch.randint(0, 256, (seer.decode_workspace_bytes(B, w.Hq, Hkv, w.d, inp.nb_max),), dtype=torch.uint8, device=DEV)
        res = []
        for rep in range(2):
            out, lse = seer.sparse_decode(inp.q, inp.k, inp.v, inp.seqlens, idx.to(DEV), cnt.to(DEV), bs, w.scale,
                                          page_table=inp.page_table, page_size=inp.page_size, out_dtype=torch.float32,
                                          workspace=ws, ragged=True)
            torch.cuda.synchronize()
            check_decode(out, lse, ref_out, ref_lse, tight=True,
                         what=f"case {case}: B={B} Hkv={Hkv} g={g} bs={bs} smax={smax} paged={w.paged} call {rep}")
            res.append((out.clone(), lse.clone()))
        assert torch.equal(res[0][0], res[1][0]) and torch.equal(res[0][1], res[1][1]), f"case {case}: the second call differs"


def test_multi_token_decode_on_random_shapes():
    """q_len new tokens per call on 24 random shapes: group sizes 1-8 with every q_len the 16-row tile
    allows, blocks of 32/64/128 tokens, contiguous and paged caches of log-uniform lengths, lists from
    empty to everything (mostly with the last block, where the causal limits among the new tokens bite),
    forced split counts and the ragged-lists hint; fp32 output at the tight bars."""
    rng = np.random.default_rng(77)
    for case in range(24):
        Hkv, g, bs = int(rng.choice([1, 2, 3, 8])), int(rng.integers(1, 9)), int(rng.choice([32, 64, 128]))
        T = int(rng.integers(1, 16 // g + 1))
        B = int(rng.choice([1, 2, 5, 17, 33]))
        smax = int(rng.choice([bs * 10, bs * 40 + 7, 2048 * 3 + 5]))
        paged = bool(rng.random() < 0.5)
        w = synth.Workload("mtr", B=B, Hq=g * Hkv, Hkv=Hkv, block_size=bs, seqlen_range=(1, smax), seqlen_dist="loguniform",
                           paged=paged, budget_tokens=0, budget_frac=0.5, seed=int(rng.integers(1, 1 << 30)))
        inp = synth.make_inputs(w, DEV)
        nb = (inp.seqlens_cpu + bs - 1) // bs
        gen = torch.Generator().manual_seed(case)
        idx, cnt = synth.random_block_lists(B, Hkv, nb, [int(rng.integers(0, int(n) + 1)) for n in nb], inp.nb_max, gen,
                                            ascending=bool(rng.random() < 0.5))
        for i in range(B):
            if rng.random() < 0.7:
                for h in range(Hkv):
                    c = int(cnt[i, h])
                    if c > 0 and (idx[i, h, :c] == int(nb[i]) - 1).sum() == 0:
                        idx[i, h, 0] = int(nb[i]) - 1
        qm = torch.randn(B, T, g * Hkv, 128, generator=gen).to(torch.bfloat16)
        kv = oracle.KVLayout(cpu(inp.k), cpu(inp.v), cpu(inp.page_table) if paged else None, inp.page_size if paged else 0)
        ref_out, ref_lse = oracle.sparse_decode_multi(qm, kv, inp.seqlens_cpu, idx, cnt, bs, w.scale)
        ragged, ns = bool(rng.random() < 0.5), int(rng.choice([0, 0, 1, 2, 3, 5]))
        seer.set_knob(1, ns)
        out, lse = seer.sparse_decode_multi(qm.to(DEV), inp.k, inp.v, inp.seqlens, idx.to(DEV), cnt.to(DEV), bs, w.scale,
                                            page_table=inp.page_table, page_size=inp.page_size, out_dtype=torch.float32,
                                            ragged=ragged)
        torch.cuda.synchronize()
        seer.set_knob(1, 0)
        R = T * g * Hkv
        check_decode(out.view(B, R, 128), lse.view(B, R), np.asarray(ref_out).reshape(B, R, 128),
                     np.asarray(ref_lse).reshape(B, R), tight=True,
                     what=f"case {case}: B={B} Hkv={Hkv} g={g} T={T} bs={bs} smax={smax} paged={paged} ragged={ragged} ns={ns}")


@pytest.mark.parametrize("seed", [5, 6])
def test_threshold_and_top_p_on_random_shapes(seed):
    """Threshold and top-p selection on 30 random shapes per seed (1-4 sequences of random lengths, 1-3 kv
    heads, every block size, caches of 3 to 3000 blocks, logits of three spreads), the threshold / the mass
    placed in the widest gap near a random target, both gate forms: indices bit-exact against the oracle."""
    rng = np.random.default_rng(seed)
    for case in range(30):
        B, Hkv, bs = int(rng.integers(1, 5)), int(rng.integers(1, 4)), int(rng.choice([16, 32, 64, 128]))
        nb_max = int(rng.choice([3, 5, 17, 64, 100, 255, 256, 257, 511, 512, 513, 700, 1024, 1500, 2048, 2500, 3000]))
        seqlens = rng.integers(2 * bs, nb_max * bs + 1, size=B).astype(np.int32)
        seqlens[rng.integers(0, B)] = nb_max * bs - int(rng.integers(0, bs))
        amp = float(rng.choice([0.3, 1.0, 3.0]))
        qg = torch.from_numpy((amp * rng.standard_normal((B, Hkv, 128))).astype(np.float32)).to(torch.bfloat16)
        kc = torch.from_numpy(rng.standard_normal((B, Hkv, nb_max, 128)).astype(np.float32)).to(torch.bfloat16)
        sl = torch.from_numpy(seqlens)
        _, _, scores = oracle.gate_select(qg, kc, sl, bs, budget_tokens=bs, max_sel=nb_max, return_scores=True)
        scores = np.asarray(scores)
        for mode in (oracle.SELECT_THRESHOLD, oracle.SELECT_TOPP):
            if mode == oracle.SELECT_THRESHOLD:
                thr = pick_threshold(scores, seqlens, bs, 128, float(rng.choice([0.05, 0.1, 0.3, 0.6])))
            else:
                thr = pick_top_p(scores, seqlens, bs, 128, 0.2, 0.95, seed=case)
            ref_idx, ref_cnt = oracle.gate_select(qg, kc, sl, bs, mode=mode, threshold=thr, max_sel=nb_max)
            for impl in (1, 2):
                seer.set_knob(3, impl)
                idx, cnt = seer.gate_select(qg.to(DEV), kc.to(DEV), sl.to(DEV), bs, mode=mode, threshold=thr, max_sel=nb_max,
                                            ragged=bool(rng.random() < 0.5))
                torch.cuda.synchronize()
                seer.set_knob(3, 0)
                check_indices(idx, cnt, ref_idx, ref_cnt,
                              what=f"case {case} mode {mode} gate form {impl}: B={B} Hkv={Hkv} bs={bs} nb_max={nb_max} thr={thr}")


def test_bursts_and_overlapping_streams():
    """200 back-to-back calls without a synchronisation, then calls overlapping on two streams (each
    with its own query set, outputs and workspace): results identical to the same calls made alone.
    The library keeps no device state between calls, so nothing can leak from one call to another."""
    w = synth.scaled(synth.CONFIGS["c2"], B=4, seqlen=64 * 96, budget_tokens=64 * 40)
    inp = synth.make_inputs(w, DEV)
    idx, cnt = gpu_gate(inp)
    seer.set_knob(1, 5)
    q2 = synth.randn_bf16(tuple(inp.q.shape), DEV, synth.generator(DEV, 77))
    o = [torch.empty(w.B, w.Hq, w.d, dtype=torch.float32, device=DEV) for _ in range(2)]
    l = [torch.empty(w.B, w.Hq, dtype=torch.float32, device=DEV) for _ in range(2)]
    ws = [torch.empty(seer.decode_workspace_bytes(w.B, w.Hq, w.Hkv, w.d, inp.max_sel), dtype=torch.uint8, device=DEV)
          for _ in range(2)]
    qs = [inp.q, q2]

    def call(r):
        seer.sparse_decode(qs[r], inp.k, inp.v, inp.seqlens, idx, cnt, w.block_size, w.scale, out=o[r], lse=l[r],
                           workspace=ws[r])

    call(0); call(1)
    torch.cuda.synchronize()
    want = [(o[r].clone(), l[r].clone()) for r in range(2)]
    ref_out, ref_lse = oracle_decode(inp, cpu(idx), cpu(cnt))
    check_decode(want[0][0], want[0][1], ref_out, ref_lse, tight=True, what="burst reference")
    for it in range(200):
        call(it % 2)
    torch.cuda.synchronize()
    for r in range(2):
        assert torch.equal(o[r], want[r][0]) and torch.equal(l[r], want[r][1]), "burst of calls changed a result"
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for r in range(2):
        o[r].zero_(); l[r].zero_()
    torch.cuda.synchronize()
    for it in range(60):
        for r in range(2):
            with torch.cuda.stream(streams[r]):
                call(r)
    torch.cuda.synchronize()
    for r in range(2):
        assert torch.equal(o[r], want[r][0]) and torch.equal(l[r], want[r][1]), "overlapping streams changed a result"


def test_gate_score_walking_kernel_on_long_caches_of_mixed_length():
    """With the mixed-lengths hint and caches longer than 8 tiles of 64 blocks the scores come from the
    kernel that walks the cache with 8 work-groups per group: lengths from a few blocks to 3000,
    a sequence ending exactly on a tile edge, block indices bit-exact in the hinted and unhinted mode."""
    w = synth.Workload("walk", B=6, Hq=8, Hkv=2, block_size=64, seqlen_range=(64, 64 * 3000), seqlen_dist="uniform",
                       budget_tokens=0, budget_frac=0.07, seed=909)
    inp = synth.make_inputs(w, DEV)
    sl = inp.seqlens_cpu.clone()
    sl[0] = 64 * 512            # ends on the boundary of the 8th tile
    sl[1] = 64 * 3 + 5          # a handful of blocks
    sl[2] = int(inp.seqlens_cpu.max())
    inp.seqlens_cpu = sl
    inp.seqlens = sl.to(DEV)
    assert inp.nb_max > 512
    ref_idx, ref_cnt = oracle_gate(inp)
    for hint in (1, 0):
        seer.set_knob(3, 1)     # score kernel + select kernel
        idx, cnt = seer.gate_select(inp.q_gate, inp.kc, inp.seqlens, w.block_size, budget_blocks=inp.budget_blocks,
                                    max_sel=inp.max_sel, ragged=bool(hint))
        torch.cuda.synchronize()
        check_indices(idx, cnt, ref_idx, ref_cnt, what=f"walk hint={hint}")
