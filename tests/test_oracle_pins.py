"""Pins for the fp64 CPU oracle (no GPU needed).

The paper prints no worked numeric example of the decode path, so the oracle is pinned to
what the mathematics fixes instead: independent dense attention, closed forms, needles,
masking equivalence, lse algebra, exact rational arithmetic, brute-force subset enumeration
and softmax invariants.  Each check below computes its expectation WITHOUT calling the oracle.
"""
import itertools
import math
from fractions import Fraction

import numpy as np
import pytest
import torch
from scipy.special import logsumexp, softmax

import oracle
from oracle import KVLayout


def bf16(x):
    return torch.as_tensor(np.asarray(x, dtype=np.float32)).to(torch.bfloat16)


def f64(t):
    return t.float().numpy().astype(np.float64)


def rand_case(seed, B=2, Hq=8, Hkv=2, d=128, S=(300, 200), b=64, k_scale=1.0):
    g = torch.Generator().manual_seed(seed)
    S_max = max(S)
    S_alloc = (S_max + b - 1) // b * b
    q = torch.randn(B, Hq, d, generator=g).to(torch.bfloat16)
    k = (torch.randn(B, Hkv, S_alloc, d, generator=g) * k_scale).to(torch.bfloat16)
    v = torch.randn(B, Hkv, S_alloc, d, generator=g).to(torch.bfloat16)
    return q, k, v, torch.tensor(S, dtype=torch.int32)


def dense_reference(q, k, v, seqlens, scale, token_mask=None):
    """Textbook softmax attention in numpy fp64 (independent of the oracle).  token_mask
    [B,Hkv,S_alloc] bool marks the tokens that take part (others get a -inf logit)."""
    qf, kf, vf = f64(q), f64(k), f64(v)
    B, Hq, d = qf.shape
    Hkv = kf.shape[1]
    g = Hq // Hkv
    out = np.zeros((B, Hq, d))
    lse = np.full((B, Hq), -np.inf)
    for i in range(B):
        S = int(seqlens[i])
        for h in range(Hq):
            hk = h // g
            x = np.float64(np.float32(scale)) * (kf[i, hk, :S] @ qf[i, h])
            if token_mask is not None:
                x = np.where(token_mask[i, hk, :S], x, -np.inf)
            if S == 0 or not np.isfinite(x).any():
                continue
            lse[i, h] = logsumexp(x)
            out[i, h] = softmax(x) @ vf[i, hk, :S]
    return out, lse


def all_blocks(B, Hkv, seqlens, b, max_sel):
    idx = np.full((B, Hkv, max_sel), -1, dtype=np.int32)
    cnt = np.zeros((B, Hkv), dtype=np.int32)
    for i in range(B):
        nb = (int(seqlens[i]) + b - 1) // b
        idx[i, :, :nb] = np.arange(nb)
        cnt[i, :] = nb
    return idx, cnt


def mask_from_blocks(idx, cnt, seqlens, b, S_alloc):
    B, Hkv, _ = idx.shape
    m = np.zeros((B, Hkv, S_alloc), dtype=bool)
    for i in range(B):
        S = int(seqlens[i])
        nb = (S + b - 1) // b
        for h in range(Hkv):
            for p in range(int(cnt[i, h])):
                j = int(idx[i, h, p])
                if 0 <= j < nb:
                    m[i, h, j * b:min((j + 1) * b, S)] = True
    return m


SCALE = 1.0 / math.sqrt(128)

# ------------------------------------------------------------------ decode


def test_all_blocks_selected_equals_dense_attention():
    q, k, v, sl = rand_case(1)
    idx, cnt = all_blocks(2, 2, sl, 64, 8)
    out, lse = oracle.sparse_decode(q, KVLayout(k, v), sl, idx, cnt, 64, SCALE)
    ro, rl = dense_reference(q, k, v, sl, SCALE)
    np.testing.assert_allclose(out, ro, rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse, rl, rtol=0, atol=1e-12)
    # the dense entry (no list) is the same thing
    out2, lse2 = oracle.sparse_decode(q, KVLayout(k, v), sl, None, None, 64, SCALE)
    np.testing.assert_array_equal(out, out2)
    np.testing.assert_array_equal(lse, lse2)


def test_query_head_to_kv_head_mapping_is_contiguous_groups():
    # kv head 0 has all-zero V, kv head 1 all-one V: heads 0..3 must give 0, heads 4..7 must give 1
    q, k, v, sl = rand_case(2, B=1, S=(128,))
    v = torch.zeros_like(v)
    v[:, 1] = 1.0
    idx, cnt = all_blocks(1, 2, sl, 64, 2)
    out, _ = oracle.sparse_decode(q, KVLayout(k, v), sl, idx, cnt, 64, SCALE)
    np.testing.assert_allclose(out[0, :4], 0.0, atol=1e-15)
    np.testing.assert_allclose(out[0, 4:], 1.0, atol=1e-13)


def test_sparse_equals_dense_with_minus_inf_on_unselected_tokens():
    q, k, v, sl = rand_case(3, S=(500, 333))
    idx = np.full((2, 2, 5), -1, dtype=np.int32)
    cnt = np.zeros((2, 2), dtype=np.int32)
    idx[0, 0, :3] = [0, 3, 7]; cnt[0, 0] = 3          # block 7 is the partial one (500 = 7*64+52)
    idx[0, 1, :2] = [6, 2]; cnt[0, 1] = 2             # unsorted on purpose
    idx[1, 0, :5] = [5, 1, 0, 4, 2]; cnt[1, 0] = 5     # 333 = 5*64+13 -> block 5 partial
    idx[1, 1, :1] = [3]; cnt[1, 1] = 1
    out, lse = oracle.sparse_decode(q, KVLayout(k, v), sl, idx, cnt, 64, SCALE)
    mask = mask_from_blocks(idx, cnt, sl, 64, k.shape[2])
    ro, rl = dense_reference(q, k, v, sl, SCALE, token_mask=mask)
    np.testing.assert_allclose(out, ro, rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse, rl, rtol=0, atol=1e-12)


def test_identical_keys_give_mean_of_selected_values_and_closed_form_lse():
    q, k, v, sl = rand_case(4, B=1, S=(300,))
    k[:] = k[0, 0, 0]                       # every key equal (all heads, all tokens)
    idx = np.array([[[1, 4, -1], [0, 2, 4]]], dtype=np.int32)   # block 4 holds 300-256 = 44 tokens
    cnt = np.array([[2, 3]], dtype=np.int32)
    out, lse = oracle.sparse_decode(q, KVLayout(k, v), sl, idx, cnt, 64, SCALE)
    vf, qf, kf = f64(v), f64(q), f64(k)
    tok = {0: list(range(64, 128)) + list(range(256, 300)),
           1: list(range(0, 64)) + list(range(128, 192)) + list(range(256, 300))}
    for h in range(8):
        hk = h // 4
        x = np.float64(np.float32(SCALE)) * (qf[0, h] @ kf[0, 0, 0])
        np.testing.assert_allclose(out[0, h], vf[0, hk, tok[hk]].mean(0), atol=1e-13)
        assert abs(lse[0, h] - (x + math.log(len(tok[hk])))) < 1e-12


@pytest.mark.parametrize("where", ["first_of_first", "last_valid_of_partial", "middle", "unselected"])
def test_needle_key_dominates_or_is_ignored(where):
    q, k, v, sl = rand_case(5, B=1, Hq=4, Hkv=1, S=(300,), k_scale=0.05)
    sel = [1, 3, 4]
    pos = {"first_of_first": 64, "last_valid_of_partial": 299, "middle": 3 * 64 + 17, "unselected": 2 * 64 + 5}[where]
    k[0, 0, pos] = (q[0, 0].float() * 40.0).to(torch.bfloat16)   # logit ~ 40*|q|^2/sqrt(d) >> others for head 0
    idx = np.array([[sel]], dtype=np.int32)
    cnt = np.array([[3]], dtype=np.int32)
    out, lse = oracle.sparse_decode(q, KVLayout(k, v), sl, idx, cnt, 64, SCALE)
    vf = f64(v)
    if where == "unselected":
        k2 = k.clone(); k2[0, 0, pos] = 0
        out2, lse2 = oracle.sparse_decode(q, KVLayout(k2, v), sl, idx, cnt, 64, SCALE)
        np.testing.assert_array_equal(out, out2)
        np.testing.assert_array_equal(lse, lse2)
    else:
        np.testing.assert_allclose(out[0, 0], vf[0, 0, pos], atol=1e-9)
        x = np.float64(np.float32(SCALE)) * (f64(q)[0, 0] @ f64(k)[0, 0, pos])
        assert abs(lse[0, 0] - x) < 1e-9
    # a token just past the sequence end is never read, even inside a selected partial block
    k3 = k.clone(); k3[0, 0, 300] = (q[0, 0].float() * 80.0).to(torch.bfloat16)
    out3, _ = oracle.sparse_decode(q, KVLayout(k3, v), sl, idx, cnt, 64, SCALE)
    np.testing.assert_array_equal(out, out3)


def test_permutation_padding_and_invalid_entries():
    q, k, v, sl = rand_case(6, B=1, S=(640,))
    a = np.array([[[0, 2, 5, 9, -1, -1], [1, 3, 4, 8, -1, -1]]], dtype=np.int32)
    cnt = np.array([[4, 4]], dtype=np.int32)
    out, lse = oracle.sparse_decode(q, KVLayout(k, v), sl, a, cnt, 64, SCALE)
    b = np.array([[[9, 0, 5, 2, 7, 7], [8, 4, 1, 3, 0, 0]]], dtype=np.int32)   # permuted; entries past nblk ignored
    out_b, lse_b = oracle.sparse_decode(q, KVLayout(k, v), sl, b, cnt, 64, SCALE)
    np.testing.assert_allclose(out, out_b, atol=1e-14)
    np.testing.assert_allclose(lse, lse_b, atol=1e-13)
    c = np.array([[[0, -1, 2, 10, 5, 9], [1, 3, 99, 4, -5, 8]]], dtype=np.int32)  # -1, 10 (== nb), 99, -5 skipped
    cnt_c = np.array([[6, 6]], dtype=np.int32)
    out_c, lse_c = oracle.sparse_decode(q, KVLayout(k, v), sl, c, cnt_c, 64, SCALE)
    np.testing.assert_allclose(out, out_c, atol=1e-14)
    np.testing.assert_allclose(lse, lse_c, atol=1e-13)


def test_lse_and_output_of_a_union_follow_the_partition_algebra():
    q, k, v, sl = rand_case(7, B=1, S=(700,))
    A = np.array([[[0, 3, 10, -1], [2, 5, -1, -1]]], dtype=np.int32); nA = np.array([[3, 2]], dtype=np.int32)
    Bm = np.array([[[1, 7, -1, -1], [4, 9, 10, -1]]], dtype=np.int32); nB = np.array([[2, 3]], dtype=np.int32)
    U = np.array([[[0, 1, 3, 7, 10, -1], [2, 4, 5, 9, 10, -1]]], dtype=np.int32); nU = np.array([[5, 5]], dtype=np.int32)
    oA, lA = oracle.sparse_decode(q, KVLayout(k, v), sl, A, nA, 64, SCALE)
    oB, lB = oracle.sparse_decode(q, KVLayout(k, v), sl, Bm, nB, 64, SCALE)
    oU, lU = oracle.sparse_decode(q, KVLayout(k, v), sl, U, nU, 64, SCALE)
    np.testing.assert_allclose(lU, np.logaddexp(lA, lB), atol=1e-12)
    wA = np.exp(lA - lU)[..., None]; wB = np.exp(lB - lU)[..., None]
    np.testing.assert_allclose(oU, wA * oA + wB * oB, atol=1e-13)


def test_empty_selection_and_empty_sequence():
    q, k, v, sl = rand_case(8, S=(128, 0))
    idx = np.full((2, 2, 2), -1, dtype=np.int32)
    cnt = np.zeros((2, 2), dtype=np.int32)
    idx[0, 1, 0] = 1; cnt[0, 1] = 1
    idx[1, :, 0] = 0; cnt[1, :] = 1          # sequence 1 has no tokens: block 0 is out of range
    out, lse = oracle.sparse_decode(q, KVLayout(k, v), sl, idx, cnt, 64, SCALE)
    assert np.all(out[0, :4] == 0) and np.all(np.isneginf(lse[0, :4]))
    assert np.all(out[1] == 0) and np.all(np.isneginf(lse[1]))
    assert np.all(np.isfinite(lse[0, 4:]))


def test_paged_layout_equals_contiguous_layout():
    q, k, v, sl = rand_case(9, S=(300, 200))
    b = 64
    B, Hkv, S_alloc, d = k.shape
    ppseq = S_alloc // b
    g = torch.Generator().manual_seed(0)
    perm = torch.randperm(B * ppseq, generator=g) + 1
    pool_k = torch.zeros(B * ppseq + 1, Hkv, b, d, dtype=torch.bfloat16)
    pool_v = torch.zeros_like(pool_k)
    pt = torch.zeros(B, ppseq, dtype=torch.int32)
    for i in range(B):
        for p in range(ppseq):
            pg = int(perm[i * ppseq + p])
            pt[i, p] = pg
            pool_k[pg] = k[i, :, p * b:(p + 1) * b]
            pool_v[pg] = v[i, :, p * b:(p + 1) * b]
    idx = np.array([[[0, 2, 4], [1, 3, 4]], [[0, 1, 3], [3, 2, -1]]], dtype=np.int32)
    cnt = np.array([[3, 3], [3, 2]], dtype=np.int32)
    o1, l1 = oracle.sparse_decode(q, KVLayout(k, v), sl, idx, cnt, b, SCALE)
    o2, l2 = oracle.sparse_decode(q, KVLayout(pool_k, pool_v, pt, b), sl, idx, cnt, b, SCALE)
    np.testing.assert_array_equal(o1, o2)
    np.testing.assert_array_equal(l1, l2)
    # page size a multiple of the block size (2 blocks per page)
    pool_k2 = torch.zeros(B * 3 + 1, Hkv, 2 * b, d, dtype=torch.bfloat16); pool_v2 = torch.zeros_like(pool_k2)
    pt2 = torch.zeros(B, 3, dtype=torch.int32)
    ids = [4, 1, 6, 2, 5, 3]
    for i in range(B):
        for p in range(3):
            pg = ids[i * 3 + p]; pt2[i, p] = pg
            seg_k = k[i, :, p * 2 * b:(p + 1) * 2 * b]; seg_v = v[i, :, p * 2 * b:(p + 1) * 2 * b]
            pool_k2[pg, :, :seg_k.shape[1]] = seg_k; pool_v2[pg, :, :seg_v.shape[1]] = seg_v
    o3, l3 = oracle.sparse_decode(q, KVLayout(pool_k2, pool_v2, pt2, 2 * b), sl, idx, cnt, b, SCALE)
    np.testing.assert_array_equal(o1, o3)
    np.testing.assert_array_equal(l1, l3)


def test_strided_cache_views_and_group_filter():
    q, k, v, sl = rand_case(10, S=(256, 256))
    big_k = torch.zeros(2, 2, 256, 256, dtype=torch.bfloat16); big_v = torch.zeros_like(big_k)
    big_k[..., :128] = k; big_v[..., :128] = v
    idx, cnt = all_blocks(2, 2, sl, 64, 4)
    o1, l1 = oracle.sparse_decode(q, KVLayout(k, v), sl, idx, cnt, 64, SCALE)
    o2, l2 = oracle.sparse_decode(q, KVLayout(big_k[..., :128], big_v[..., :128]), sl, idx, cnt, 64, SCALE)
    np.testing.assert_array_equal(o1, o2)
    filt = np.array([[1, 0], [0, 1]], dtype=np.uint8)
    o3, l3 = oracle.sparse_decode(q, KVLayout(k, v), sl, idx, cnt, 64, SCALE, group_filter=filt)
    np.testing.assert_array_equal(o3[0, :4], o1[0, :4]); assert np.isnan(o3[0, 4:]).all()
    np.testing.assert_array_equal(o3[1, 4:], o1[1, 4:]); assert np.isnan(l3[1, :4]).all()


# -------------------------------------------------------------------- gate


def gate_case(seed, B=2, Hkv=2, Dg=128, nb_max=12, integer=False):
    g = torch.Generator().manual_seed(seed)
    if integer:      # small integers: exact in bf16, many exact ties between scores
        qg = torch.randint(-2, 3, (B, Hkv, Dg), generator=g).to(torch.bfloat16)
        kc = torch.randint(-1, 2, (B, Hkv, nb_max, Dg), generator=g).to(torch.bfloat16)
    else:
        qg = torch.randn(B, Hkv, Dg, generator=g).to(torch.bfloat16)
        kc = torch.randn(B, Hkv, nb_max, Dg, generator=g).to(torch.bfloat16)
    return qg, kc


def exact_scores(qg, kc, i, h, n):
    """Exact rational dot products (bf16 values are dyadic rationals)."""
    qv = [Fraction(float(x)) for x in qg[i, h].float().tolist()]
    out = []
    for j in range(n):
        kv = [Fraction(float(x)) for x in kc[i, h, j].float().tolist()]
        out.append(sum(a * b for a, b in zip(qv, kv)))
    return out


def test_gate_score_is_the_exact_dot_product():
    qg, kc = gate_case(11)
    sl = torch.tensor([12 * 64, 7 * 64 + 5], dtype=torch.int32)
    _, _, scores = oracle.gate_select(qg, kc, sl, 64, budget_tokens=64, max_sel=12, return_scores=True)
    for i, nfull in ((0, 12), (1, 7)):
        for h in range(2):
            ex = exact_scores(qg, kc, i, h, nfull)
            for j in range(nfull):
                assert Fraction(float(scores[i, h, j])) == ex[j], (i, h, j)
            assert np.isnan(scores[i, h, nfull:]).all()      # stale / absent entries are never scored
    # a transposed or mis-strided read would not survive this: kc given as a strided view
    wide = torch.zeros(2, 2, 12, 256, dtype=torch.bfloat16); wide[..., 128:] = kc
    _, _, s2 = oracle.gate_select(qg, wide[..., 128:], sl, 64, budget_tokens=64, max_sel=12, return_scores=True)
    np.testing.assert_array_equal(scores, s2)


def brute_force_topk(scores, k):
    """Among all k-subsets: the largest score sum, and of those the lexicographically smallest
    sorted index tuple.  Exact arithmetic on Fractions."""
    n = len(scores)
    best = None
    for comb in itertools.combinations(range(n), k):
        key = (-sum(scores[j] for j in comb), comb)
        if best is None or key < best:
            best = key
    return list(best[1]) if best else []


@pytest.mark.parametrize("integer", [False, True])
def test_topk_equals_brute_force_subset_enumeration(integer):
    qg, kc = gate_case(12, B=3, Hkv=2, nb_max=9, integer=integer)
    b = 64
    sl = torch.tensor([9 * b, 6 * b + 1, 8 * b + 63], dtype=torch.int32)
    for budget_blocks in (1, 2, 4, 6):
        idx, cnt = oracle.gate_select(qg, kc, sl, b, budget_tokens=budget_blocks * b, max_sel=9)
        for i in range(3):
            S = int(sl[i]); nfull = S // b; nb = (S + b - 1) // b
            partial = nb > nfull
            k = min(budget_blocks, nb)
            for h in range(2):
                ex = exact_scores(qg, kc, i, h, nfull)
                if partial:
                    want = sorted(brute_force_topk(ex, min(k - 1, nfull)) + [nb - 1])
                else:
                    want = brute_force_topk(ex, k)
                got = idx[i, h, :cnt[i, h]].tolist()
                assert got == want, (budget_blocks, i, h, got, want)
                assert (idx[i, h, cnt[i, h]:] == -1).all()
                assert cnt[i, h] == len(want)


def test_topk_edge_rules():
    qg, kc = gate_case(13, B=1, Hkv=1, nb_max=10)
    b = 64
    sl = torch.tensor([10 * b], dtype=torch.int32)
    s = np.array([float(x) for x in exact_scores(qg, kc, 0, 0, 10)])
    idx, cnt = oracle.gate_select(qg, kc, sl, b, budget_tokens=1, max_sel=10)        # 1 token -> 1 block -> argmax
    assert cnt[0, 0] == 1 and idx[0, 0, 0] == int(np.argmax(s))
    idx, cnt = oracle.gate_select(qg, kc, sl, b, budget_tokens=b + 1, max_sel=10)    # rounds up to 2 blocks
    assert cnt[0, 0] == 2
    idx, cnt = oracle.gate_select(qg, kc, sl, b, budget_tokens=10 ** 6, max_sel=10)  # k >= nb -> everything
    assert idx[0, 0].tolist() == list(range(10))
    # all scores equal -> the k lowest indices
    kc_eq = kc.clone(); kc_eq[0, 0, :] = kc[0, 0, 3]
    idx, cnt = oracle.gate_select(qg, kc_eq, sl, b, budget_tokens=4 * b, max_sel=10)
    assert idx[0, 0, :4].tolist() == [0, 1, 2, 3] and cnt[0, 0] == 4
    # duplicated best entry: the lower index wins at k = 1
    kc_dup = kc.clone(); best = int(np.argmax(s)); other = (best + 5) % 10
    kc_dup[0, 0, other] = kc[0, 0, best]
    idx, cnt = oracle.gate_select(qg, kc_dup, sl, b, budget_tokens=b, max_sel=10)
    assert idx[0, 0, 0] == min(best, other)
    # per-sequence block budgets override the token budget; 0 selects nothing
    idx, cnt = oracle.gate_select(qg, kc, sl, b, budget_tokens=5 * b, budget_blocks=np.array([3], dtype=np.int32), max_sel=10)
    assert cnt[0, 0] == 3 and sorted(np.argsort(-s, kind="stable")[:3].tolist()) == idx[0, 0, :3].tolist()
    idx, cnt = oracle.gate_select(qg, kc, sl, b, budget_blocks=np.array([0], dtype=np.int32), max_sel=10)
    assert cnt[0, 0] == 0 and (idx == -1).all()
    # partial last block: always present, inside the budget; its own (stale) cache entry is irrelevant
    sl_p = torch.tensor([9 * b + 7], dtype=torch.int32)
    for kb in (1, 2, 5, 10, 50):
        idx, cnt = oracle.gate_select(qg, kc, sl_p, b, budget_tokens=kb * b, max_sel=10)
        n = int(cnt[0, 0])
        assert n == min(kb, 10) and idx[0, 0, n - 1] == 9
        want = sorted(np.argsort(-s[:9], kind="stable")[:n - 1].tolist()) + [9]
        assert idx[0, 0, :n].tolist() == want
        kc_stale = kc.clone(); kc_stale[0, 0, 9] = 100.0
        idx2, cnt2 = oracle.gate_select(qg, kc_stale, sl_p, b, budget_tokens=kb * b, max_sel=10)
        np.testing.assert_array_equal(idx, idx2)
    # empty sequence / shorter than one block
    idx, cnt = oracle.gate_select(qg, kc, torch.tensor([0], dtype=torch.int32), b, budget_tokens=4 * b, max_sel=10)
    assert cnt[0, 0] == 0
    idx, cnt = oracle.gate_select(qg, kc, torch.tensor([5], dtype=torch.int32), b, budget_tokens=4 * b, max_sel=10)
    assert cnt[0, 0] == 1 and idx[0, 0, 0] == 0


def test_threshold_mode_matches_independent_softmax_and_its_invariants():
    qg, kc = gate_case(14, B=2, Hkv=2, nb_max=40)
    b = 64
    sl = torch.tensor([40 * b, 33 * b + 9], dtype=torch.int32)
    qf, kf = f64(qg), f64(kc)
    prev = None
    for tau in (0.0, 1e-4, 2e-3, 6e-3, 0.02, 0.1, 0.5, 1.0):
        idx, cnt = oracle.gate_select(qg, kc, sl, b, mode=oracle.SELECT_THRESHOLD, threshold=tau, max_sel=40)
        for i, (nfull, partial) in enumerate(((40, False), (33, True))):
            for h in range(2):
                s = kf[i, h, :nfull] @ qf[i, h]
                P = softmax(s / math.sqrt(128))
                assert abs(P.sum() - 1) < 1e-12
                want = [j for j in range(nfull) if P[j] > tau] + ([33] if partial else [])
                assert idx[i, h, :cnt[i, h]].tolist() == want, (tau, i, h)
                assert (idx[i, h, cnt[i, h]:] == -1).all()
        if prev is not None:
            assert (cnt <= prev).all()           # selection shrinks as tau grows
        prev = cnt.copy()
    # tau >= 1 keeps only the forced block; tau below every probability keeps all full blocks
    assert prev.tolist() == [[0, 0], [1, 1]]
    idx, cnt = oracle.gate_select(qg, kc, sl, b, mode=oracle.SELECT_THRESHOLD, threshold=-1.0, max_sel=40)
    assert cnt.tolist() == [[40, 40], [34, 34]]
    # strict comparison: four equal scores have probability exactly 1/4 each
    kc4 = kc[:, :, :4].clone(); kc4[:] = kc[0, 0, 0]
    sl4 = torch.tensor([4 * b, 4 * b], dtype=torch.int32)
    _, c = oracle.gate_select(qg, kc4, sl4, b, mode=oracle.SELECT_THRESHOLD, threshold=0.25, max_sel=4)
    assert (c == 0).all()
    _, c = oracle.gate_select(qg, kc4, sl4, b, mode=oracle.SELECT_THRESHOLD, threshold=0.2499999, max_sel=4)
    assert (c == 4).all()
    # too small a list is reported, not silently truncated
    with pytest.raises(ValueError):
        oracle.gate_select(qg, kc, sl, b, mode=oracle.SELECT_THRESHOLD, threshold=-1.0, max_sel=8)


def test_topk_on_raw_scores_equals_topk_on_softmaxed_scores():
    # Sec. 3.1: the token-budget method needs no softmax because softmax is monotone
    qg, kc = gate_case(15, B=1, Hkv=2, nb_max=64)
    b = 64
    sl = torch.tensor([64 * b], dtype=torch.int32)
    idx, cnt = oracle.gate_select(qg, kc, sl, b, budget_tokens=16 * b, max_sel=16)
    qf, kf = f64(qg), f64(kc)
    for h in range(2):
        P = softmax((kf[0, h] @ qf[0, h]) / math.sqrt(128))
        want = sorted(np.argsort(-P, kind="stable")[:16].tolist())
        assert idx[0, h].tolist() == want


def test_compression_cache_is_one_128th_of_the_kv_cache_at_block_64():
    # Sec. 3.2: with b = 64 and d_gate = d the K Compression Cache is 1/128 of the KV bytes
    d = dg = 128; b = 64
    kv_bytes_per_block = 2 * b * d * 2
    kc_bytes_per_block = dg * 2
    assert kv_bytes_per_block == 128 * kc_bytes_per_block


def test_bf16_inputs_are_read_exactly_including_subnormal_and_negative_zero():
    vals = np.array([0.0, -0.0, 1.0, -1.5, 3.0e-39, 2.0 ** -126, 65280.0, -3.3895314e38], dtype=np.float32)
    t = torch.tensor(vals).to(torch.bfloat16)
    qg = torch.zeros(1, 1, 128, dtype=torch.bfloat16); qg[0, 0, :8] = 1.0
    kc = torch.zeros(1, 1, 8, 128, dtype=torch.bfloat16)
    for j in range(8):
        kc[0, 0, j, j] = t[j]
    _, _, s = oracle.gate_select(qg, kc, torch.tensor([8 * 64], dtype=torch.int32), 64, budget_tokens=64,
                                 max_sel=8, return_scores=True)
    np.testing.assert_array_equal(s[0, 0], t.float().numpy().astype(np.float64))


def test_top_p_mode_matches_sorted_cumulative_probabilities():
    """Nucleus selection (the adaptive-sparsity direction of Sec. 6.2): smallest prefix of the
    score-descending order whose softmax mass reaches p."""
    qg, kc = gate_case(16, B=2, Hkv=2, nb_max=50)
    b = 64
    sl = torch.tensor([50 * b, 41 * b + 3], dtype=torch.int32)
    qf, kf = f64(qg), f64(kc)
    prev = None
    for p in (0.0, 0.05, 0.3, 0.5, 0.9, 0.999, 1.0, 1.5):
        idx, cnt = oracle.gate_select(qg, kc, sl, b, mode=oracle.SELECT_TOPP, threshold=p, max_sel=50)
        for i, (nfull, partial) in enumerate(((50, False), (41, True))):
            for h in range(2):
                s = kf[i, h, :nfull] @ qf[i, h]
                P = softmax(s / math.sqrt(128))
                order = np.lexsort((np.arange(nfull), -s))            # score descending, index ascending
                cum = np.cumsum(P[order])
                k = int(np.searchsorted(cum, p, side="left")) + 1      # first prefix with cum >= p
                k = min(max(k, 1), nfull)
                # keep away from razor edges where summation order could matter
                assert p <= 0 or p > 1 or k == nfull or min(abs(cum[k - 1] - p), abs(cum[k - 2] - p) if k > 1 else 1) > 1e-9
                want = sorted(order[:k].tolist()) + ([41] if partial else [])
                assert idx[i, h, :cnt[i, h]].tolist() == want, (p, i, h)
        if prev is not None:
            assert (cnt >= prev).all()           # the nucleus grows with p
        prev = cnt.copy()
    assert prev.tolist() == [[50, 50], [42, 42]]  # p beyond the total mass keeps every block
    idx, cnt = oracle.gate_select(qg, kc, sl, b, mode=oracle.SELECT_TOPP, threshold=0.0, max_sel=50)
    assert cnt.tolist() == [[1, 1], [2, 2]]       # at least the best block (plus the forced partial one)
    # equal scores: probability 1/8 each, p = 0.5 needs exactly 4, the lowest indices
    kc8 = kc[:, :, :8].clone(); kc8[:] = kc[0, 0, 0]
    idx, cnt = oracle.gate_select(qg, kc8, torch.tensor([8 * b, 8 * b], dtype=torch.int32), b, mode=oracle.SELECT_TOPP,
                                  threshold=0.5, max_sel=8)
    assert (cnt == 4).all() and idx[0, 0, :4].tolist() == [0, 1, 2, 3]
    # p = 1 is the whole mass, i.e. every full block, also when one block dominates so strongly that a
    # rounded running sum touches 1.0 after the first block (5 blocks: scores 512, 0, 0, 0, 0 -> the
    # first probability is 1 - 4e-20, which is 1.0 in fp64); just below 1 the nucleus is that one block
    qd = torch.zeros(1, 1, 128, dtype=torch.bfloat16); qd[0, 0, 0] = 32.0
    kd = torch.zeros(1, 1, 6, 128, dtype=torch.bfloat16); kd[0, 0, 0, 0] = 16.0
    kd[0, 0, 5] = 99.0                                                 # stale entry of the partial sixth block: never read
    sl5 = torch.tensor([5 * b + 7], dtype=torch.int32)
    idx, cnt = oracle.gate_select(qd, kd, sl5, b, mode=oracle.SELECT_TOPP, threshold=1.0, max_sel=6)
    assert cnt.tolist() == [[6]] and idx[0, 0].tolist() == [0, 1, 2, 3, 4, 5]
    idx, cnt = oracle.gate_select(qd, kd, sl5, b, mode=oracle.SELECT_TOPP, threshold=0.999999, max_sel=6)
    assert cnt.tolist() == [[2]] and idx[0, 0, :2].tolist() == [0, 5]


def test_multi_token_decode_is_a_stack_of_single_token_decodes_and_causal():
    """Query t of T new tokens == single-token decode of the sequence cut at that token (same list);
    and independently: dense causal attention over the last T positions when every block is listed."""
    q, k, v, sl = rand_case(17, B=2, S=(300, 135))
    T = 3
    g = torch.Generator().manual_seed(3)
    qm = torch.randn(2, T, 8, 128, generator=g).to(torch.bfloat16)
    idx = np.array([[[0, 2, 4, -1, -1], [1, 3, 4, -1, -1]], [[0, 1, 2, -1, -1], [2, 0, -1, -1, -1]]], dtype=np.int32)
    cnt = np.array([[3, 3], [3, 2]], dtype=np.int32)
    out, lse = oracle.sparse_decode_multi(qm, KVLayout(k, v), sl, idx, cnt, 64, SCALE)
    for t in range(T):
        cut = sl - (T - 1 - t)
        o1, l1 = oracle.sparse_decode(qm[:, t].contiguous(), KVLayout(k, v), cut, idx, cnt, 64, SCALE)
        np.testing.assert_allclose(out[:, t], o1, rtol=0, atol=1e-13)
        np.testing.assert_allclose(lse[:, t], l1, rtol=0, atol=1e-12)
    # all blocks listed: textbook causal attention of the last T tokens (independent numpy)
    idx_all, cnt_all = all_blocks(2, 2, sl, 64, 5)
    out, lse = oracle.sparse_decode_multi(qm, KVLayout(k, v), sl, idx_all, cnt_all, 64, SCALE)
    for t in range(T):
        ro, rl = dense_reference(qm[:, t], k, v, sl - (T - 1 - t), SCALE)
        np.testing.assert_allclose(out[:, t], ro, rtol=0, atol=1e-13)
        np.testing.assert_allclose(lse[:, t], rl, rtol=0, atol=1e-12)
    # a later token never leaks into an earlier query: changing the last key/value leaves queries 0..T-2 alone
    k2, v2 = k.clone(), v.clone()
    k2[0, :, 299] = 3.0; v2[0, :, 299] = -5.0
    out2, _ = oracle.sparse_decode_multi(qm, KVLayout(k2, v2), sl, idx_all, cnt_all, 64, SCALE)
    np.testing.assert_array_equal(out2[0, :T - 1], out[0, :T - 1])
    assert np.abs(out2[0, T - 1] - out[0, T - 1]).max() > 1e-3
    # more new tokens than the sequence holds: the earliest queries see nothing
    out3, lse3 = oracle.sparse_decode_multi(qm, KVLayout(k, v), torch.tensor([2, 1], dtype=torch.int32), idx_all, cnt_all, 64, SCALE)
    assert np.isneginf(lse3[0, 0]).all() and np.isfinite(lse3[0, 1]).all() and np.isneginf(lse3[1, :2]).all()
