"""Pins for the oracle's training-side ground truth (Sec. 2.3: column-wise max pooling of the causal
attention map per block, max over the query heads of a kv head, normalised to sum 1) - CPU only.
Expectations are closed forms, properties, or come from the separately written decode oracle."""
import math

import numpy as np
import pytest
import torch

import oracle

D = 128


def rand_case(seed, B=2, T=150, Hq=4, Hkv=2):
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(B, T, Hq, D, generator=g).to(torch.bfloat16)
    k = torch.randn(B, Hkv, T, D, generator=g).to(torch.bfloat16)
    v = torch.randn(B, Hkv, T, D, generator=g).to(torch.bfloat16)
    return q, k, v


def test_zero_queries_give_prefix_means_and_uniform_ground_truth():
    q, k, v = rand_case(1, B=1, T=100, Hq=4, Hkv=2)
    q.zero_()
    b = 16
    out, lse, gt = oracle.attn_ground_truth(q, k, v, b, 0.3)
    vd = v.double().numpy()
    prefix = np.cumsum(vd, axis=2) / np.arange(1, 101)[None, None, :, None]      # [1,Hkv,T,D]
    for h in range(4):
        np.testing.assert_allclose(out[0, :, h], prefix[0, h // 2], rtol=0, atol=1e-12)
        np.testing.assert_allclose(lse[0, :, h], np.log(np.arange(1, 101)), rtol=0, atol=1e-12)
    nb = 7
    assert gt.shape == (1, 2, 100, nb)
    for t in range(100):
        nvis = t // b + 1                      # blocks that hold at least one key s <= t
        want = np.zeros(nb)
        want[:nvis] = 1.0 / nvis
        np.testing.assert_allclose(gt[0, 0, t], want, rtol=0, atol=1e-14)
        np.testing.assert_allclose(gt[0, 1, t], want, rtol=0, atol=1e-14)


def test_identical_keys_are_uniform_whatever_the_query():
    q, k, v = rand_case(2, B=1, T=40, Hq=2, Hkv=1)
    k[:] = k[:, :, :1]
    out, lse, gt = oracle.attn_ground_truth(q, k, v, 8, 0.11)
    for t in (0, 7, 8, 39):
        nvis = t // 8 + 1
        np.testing.assert_allclose(gt[0, 0, t, :nvis], 1.0 / nvis, rtol=0, atol=1e-13)
        assert (gt[0, 0, t, nvis:] == 0).all()
        np.testing.assert_allclose(out[0, t, 0], v.double()[0, 0, :t + 1].mean(0).numpy(), rtol=0, atol=1e-12)


def test_needle_keys_closed_form_with_two_heads_pointing_at_different_blocks():
    # All keys zero except one needle per head direction: head 0 looks along e_0, head 1 along e_1.
    # Needle A (feature 0) at position 21, needle B (feature 1) at position 50; block size 16.
    T, b = 70, 16
    a = 4.0                                    # bf16-exact
    scale = 0.25                               # logit of a needle = scale * a * a = 4
    q = torch.zeros(1, T, 2, D, dtype=torch.bfloat16)
    q[0, :, 0, 0] = a
    q[0, :, 1, 1] = a
    k = torch.zeros(1, 1, T, D, dtype=torch.bfloat16)
    k[0, 0, 21, 0] = a
    k[0, 0, 50, 1] = a
    v = torch.randn(1, 1, T, D, generator=torch.Generator().manual_seed(3)).to(torch.bfloat16)
    out, lse, gt = oracle.attn_ground_truth(q, k, v, b, scale)
    E = math.exp(4.0)
    vd = v.double().numpy()[0, 0]
    for t in (0, 20, 21, 22, 31, 32, 49, 50, 69):
        n = t + 1
        pa = [(E if t >= 21 else 1.0) / ((E + n - 1) if t >= 21 else n), 1.0 / ((E + n - 1) if t >= 21 else n)]
        pb = [(E if t >= 50 else 1.0) / ((E + n - 1) if t >= 50 else n), 1.0 / ((E + n - 1) if t >= 50 else n)]
        # per-head column maxima per block, then the head-wise maximum
        raw = np.zeros(5)
        for j in range(t // b + 1):
            ca = pa[0] if (t >= 21 and j == 21 // b) else pa[1]
            cb = pb[0] if (t >= 50 and j == 50 // b) else pb[1]
            raw[j] = max(ca, cb)
        np.testing.assert_allclose(gt[0, 0, t], raw / raw.sum(), rtol=1e-13, atol=0)
        # outputs of both heads
        za = (E + n - 1) if t >= 21 else n
        wa = np.ones(n); wa[21:22] = E if t >= 21 else 1.0
        np.testing.assert_allclose(out[0, t, 0], (wa[:, None] * vd[:n]).sum(0) / za, rtol=0, atol=1e-12)
        np.testing.assert_allclose(lse[0, t, 0], math.log(za), rtol=0, atol=1e-12)
        zb = (E + n - 1) if t >= 50 else n
        np.testing.assert_allclose(lse[0, t, 1], math.log(zb), rtol=0, atol=1e-12)


def test_out_and_lse_match_the_decode_oracle_position_by_position():
    q, k, v = rand_case(4, B=2, T=90, Hq=4, Hkv=2)
    b = 32
    out, lse, gt = oracle.attn_ground_truth(q, k, v, b, 0.09)
    for t in (0, 1, 31, 32, 63, 64, 89):
        sl = torch.full((2,), t + 1, dtype=torch.int32)
        o1, l1 = oracle.sparse_decode(q[:, t].contiguous(), oracle.KVLayout(k, v), sl, None, None, b, 0.09)
        np.testing.assert_allclose(out[:, t], o1, rtol=0, atol=1e-12)
        np.testing.assert_allclose(lse[:, t], l1, rtol=0, atol=1e-12)


def test_pooling_over_blocks_and_heads_follows_from_block_size_one_single_head_rows():
    # With block size 1 and one head the ground truth is the causal softmax row P itself (pinned by
    # the last test of this file through out = P v with linearly independent value rows).  Any other
    # block size / grouping must equal max-pooling those rows: over the keys of a block, then over the
    # heads of the group, then normalising.
    q, k, v = rand_case(5, B=2, T=70, Hq=4, Hkv=2)
    P = np.zeros((2, 4, 70, 70))
    for h in range(4):
        hk = h // 2
        _, _, p1 = oracle.attn_ground_truth(q[:, :, h:h + 1].contiguous(), k[:, hk:hk + 1], v[:, hk:hk + 1], 1, 0.13)
        P[:, h] = p1[:, 0]
    for b in (16, 32, 7):
        _, _, gt = oracle.attn_ground_truth(q, k, v, b, 0.13)
        nb = (70 + b - 1) // b
        for hk in range(2):
            grp = np.maximum(P[:, 2 * hk], P[:, 2 * hk + 1])                   # [B,T,T]
            raw = np.stack([grp[:, :, j * b:(j + 1) * b].max(-1) for j in range(nb)], axis=-1)
            np.testing.assert_allclose(gt[:, hk], raw / raw.sum(-1, keepdims=True), rtol=1e-12, atol=0)


def test_rows_sum_to_one_are_causal_and_padding_rows_are_empty():
    q, k, v = rand_case(6, B=3, T=130, Hq=6, Hkv=2)
    b = 32
    sl = torch.tensor([130, 77, 1], dtype=torch.int32)
    out, lse, gt = oracle.attn_ground_truth(q, k, v, b, 0.09, seqlens=sl)
    nb = 5
    for i in range(3):
        S = int(sl[i])
        np.testing.assert_allclose(gt[i, :, :S].sum(-1), 1.0, rtol=0, atol=1e-13)
        for t in range(S):
            nvis = t // b + 1
            assert (gt[i, :, t, :nvis] > 0).all() and (gt[i, :, t, nvis:] == 0).all()
        assert (gt[i, :, S:] == 0).all() and (out[i, S:] == 0).all() and np.isneginf(lse[i, S:]).all()
    # a real row does not depend on what lies after it or on the padding
    out2, lse2, gt2 = oracle.attn_ground_truth(q[:, :77].contiguous(), k[:, :, :77], v[:, :, :77], b, 0.09)
    np.testing.assert_array_equal(gt2[1, :, :, :3], gt[1, :, :77, :3])
    np.testing.assert_array_equal(out2[1], out[1, :77])


def test_shuffling_keys_inside_a_block_changes_nothing_for_later_queries():
    q, k, v = rand_case(7, B=1, T=96, Hq=4, Hkv=2)
    b = 16
    perm = torch.arange(96)
    perm[32:48] = 32 + torch.randperm(16, generator=torch.Generator().manual_seed(1))
    out, lse, gt = oracle.attn_ground_truth(q, k, v, b, 0.09)
    out2, lse2, gt2 = oracle.attn_ground_truth(q, k[:, :, perm].contiguous(), v[:, :, perm].contiguous(), b, 0.09)
    np.testing.assert_allclose(gt2[0, :, 48:], gt[0, :, 48:], rtol=1e-12, atol=0)
    np.testing.assert_allclose(out2[0, 48:], out[0, 48:], rtol=0, atol=1e-12)
    assert np.abs(gt2[0, :, 33:47] - gt[0, :, 33:47]).max() > 1e-3      # inside the block it matters


def test_block_size_one_is_the_attention_row_itself_and_one_block_is_all_mass():
    q, k, v = rand_case(8, B=1, T=24, Hq=1, Hkv=1)
    out, lse, gt = oracle.attn_ground_truth(q, k, v, 1, 0.09)
    # block size 1, one head: gt is the causal softmax row (already sums to 1) -> out = gt @ v
    np.testing.assert_allclose(np.einsum("ts,sc->tc", gt[0, 0], v.double().numpy()[0, 0]), out[0, :, 0],
                               rtol=0, atol=1e-12)
    _, _, gt_all = oracle.attn_ground_truth(q, k, v, 64, 0.09)
    np.testing.assert_array_equal(gt_all[0, 0, :, 0], np.ones(24))
