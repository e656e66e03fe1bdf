"""Pins for the oracle's AttnGate front-end (Eq. 1a / 1b: query-head reduction, pooled-key
projection, RoPE) - CPU only.  Expectations are computed here with numpy / torch fp64 and complex
arithmetic, never by calling the oracle."""
import math
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
import synth

D = 128
DG = 128


def f64(t):
    return t.float().numpy().astype(np.float64)


def rope_complex(y, cos_row, sin_row):
    """Rotate-half RoPE as a complex multiplication: (y_c + i y_{c+D/2}) * e^{i angle_c}."""
    half = y.shape[-1] // 2
    z = (y[..., :half] + 1j * y[..., half:]) * (cos_row.astype(np.float64) + 1j * sin_row.astype(np.float64))
    return np.concatenate([z.real, z.imag], axis=-1)


def case(seed, B=3, Hq=8, Hkv=2, S=(640, 200, 64), b=64):
    g = torch.Generator().manual_seed(seed)
    S_alloc = (max(S) + b - 1) // b * b
    q = torch.randn(B, Hq, D, generator=g).to(torch.bfloat16)
    k = torch.randn(B, Hkv, S_alloc, D, generator=g).to(torch.bfloat16)
    wq = (torch.randn(Hkv, DG, (Hq // Hkv) * D, generator=g) / math.sqrt((Hq // Hkv) * D)).to(torch.bfloat16)
    wk = (torch.randn(Hkv, DG, 3 * D, generator=g) / math.sqrt(3 * D)).to(torch.bfloat16)
    return q, k, wq, wk, torch.tensor(S, dtype=torch.int32)


def test_q_branch_equals_matmul_then_complex_rotation_at_the_current_position():
    q, k, wq, wk, sl = case(1)
    cos, sin = synth.rope_tables(700, DG)
    out, bits = oracle.gate_q(q, wq, cos, sin, sl)
    qf, wf = f64(q), f64(wq)
    for i in range(3):
        pos = int(sl[i]) - 1
        for h in range(2):
            x = qf[i, h * 4:(h + 1) * 4].reshape(-1)          # heads of the group, head-major
            want = rope_complex(wf[h] @ x, cos[pos].numpy(), sin[pos].numpy())
            np.testing.assert_allclose(out[i, h], want, rtol=0, atol=1e-12)
    # the rounded output is the unrounded one rounded to bf16
    back = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).float().numpy()
    assert np.all(np.abs(back - out) <= np.abs(out) * 2.0 ** -8 + 1e-40)


def test_q_branch_special_weights_identity_mean_and_position_zero():
    q, k, wq, wk, sl = case(2, B=2, S=(1, 1))
    cos, sin = synth.rope_tables(4, DG)
    eye = torch.eye(D)
    # picks head r of each group; position 0 is the identity rotation
    for r in range(4):
        w = torch.zeros(2, DG, 4 * D)
        w[:, :, r * D:(r + 1) * D] = eye
        out, bits = oracle.gate_q(q, w.to(torch.bfloat16), cos, sin, sl)
        for h in range(2):
            np.testing.assert_array_equal(out[:, h], f64(q)[:, h * 4 + r])
            np.testing.assert_array_equal(bits[:, h], q[:, h * 4 + r].view(torch.int16).numpy().view(np.uint16))
    # 1/g on every head = mean of the group's query heads (the tiny benchmark config builds q_gate this way)
    w = torch.cat([eye * 0.25] * 4, dim=1).expand(2, DG, 4 * D).contiguous().to(torch.bfloat16)
    out, _ = oracle.gate_q(q, w, cos, sin, sl)
    np.testing.assert_allclose(out, q.double().view(2, 2, 4, D).mean(2).numpy(), rtol=0, atol=1e-15)


def test_rope_keeps_norms_and_dot_products_depend_on_relative_position_only():
    q, k, wq, wk, _ = case(3, B=1, Hq=4, Hkv=1, S=(64,))
    cos, sin = synth.rope_tables(3000, DG)
    eye = torch.zeros(1, DG, 4 * D); eye[0, :, :D] = torch.eye(D)
    eye = eye.to(torch.bfloat16)
    outs = {}
    for pos in (0, 1, 17, 1000, 1017, 2999):
        o, _ = oracle.gate_q(q, eye, cos, sin, torch.tensor([pos + 1], dtype=torch.int32))
        outs[pos] = o[0, 0]
        assert abs(np.linalg.norm(o[0, 0]) - np.linalg.norm(f64(q)[0, 0])) < 1e-5
    q2 = q.clone(); q2[0, 0] = k[0, 0, 5]
    outs2 = {}
    for pos in (0, 17, 1000, 1017):
        o, _ = oracle.gate_q(q2, eye, cos, sin, torch.tensor([pos + 1], dtype=torch.int32))
        outs2[pos] = o[0, 0]
    # <R(p+17) a, R(p) b> is the same for p = 0 and p = 1000 (tables are fp32, hence 1e-4)
    assert abs(outs[17] @ outs2[0] - outs[1017] @ outs2[1000]) < 2e-4
    assert abs(outs[17] @ outs2[0] - outs[0] @ outs2[0]) > 1e-2          # and it does depend on the offset


def test_k_branch_equals_pool_concat_matmul_rotation_at_block_start():
    q, k, wq, wk, sl = case(4)
    b = 64
    cos, sin = synth.rope_tables(700, DG)
    out, bits = oracle.kc_update(k, wk, cos, sin, sl, b, 10)
    kf, wf = f64(k), f64(wk)
    for i in range(3):
        nfull = int(sl[i]) // b
        for h in range(2):
            for j in range(10):
                if j >= nfull:
                    assert np.isnan(out[i, h, j]).all()       # partial / absent blocks get no entry
                    continue
                X = kf[i, h, j * b:(j + 1) * b]
                u = np.concatenate([X.max(0), X.min(0), X.mean(0)])
                want = rope_complex(wf[h] @ u, cos[j * b].numpy(), sin[j * b].numpy())
                np.testing.assert_allclose(out[i, h, j], want, rtol=0, atol=1e-12)
    back = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).float().numpy()
    ok = ~np.isnan(out)
    assert np.all(np.abs(back[ok] - out[ok]) <= np.abs(out[ok]) * 2.0 ** -8 + 1e-40)


def test_k_branch_special_weights_give_block_max_min_and_mean():
    q, k, wq, wk, sl = case(5, B=2, S=(256, 130))
    b = 64
    ones = torch.ones(300, DG // 2); zeros = torch.zeros(300, DG // 2)     # no rotation
    eye = torch.eye(D)
    z = torch.zeros(D, D)
    kd = k.double()
    for which, ref in ((0, lambda X: X.amax(2)), (1, lambda X: X.amin(2)), (2, lambda X: X.mean(2))):
        blocks = [z, z, z]; blocks[which] = eye
        w = torch.cat(blocks, dim=1).expand(2, DG, 3 * D).contiguous().to(torch.bfloat16)
        out, _ = oracle.kc_update(k, w, ones, zeros, sl, b, 4)
        np.testing.assert_allclose(out[0], ref(kd[0, :, :256].view(2, 4, b, D)).numpy(), rtol=0, atol=1e-15)
        np.testing.assert_allclose(out[1, :, :2], ref(kd[1, :, :128].view(2, 2, b, D)).numpy(), rtol=0, atol=1e-15)
        assert np.isnan(out[1, :, 2:]).all()
    # the mean case is the recipe of the tiny benchmark config (block mean of K as the gate input)
    w = torch.cat([z, z, eye], dim=1).expand(2, DG, 3 * D).contiguous().to(torch.bfloat16)
    out, bits = oracle.kc_update(k[:1, :, :256], w, ones, zeros, sl[:1], b, 4)
    want = synth._block_means(k[:1, :, :256], b, 4)
    got = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16)
    assert (got.float() - want.float()).abs().max() <= 2.0 ** -8 * want.float().abs().max()


def test_k_branch_block_ranges_and_paged_layout():
    q, k, wq, wk, sl = case(6, B=2, S=(640, 320))
    b = 64
    cos, sin = synth.rope_tables(700, DG)
    full, full_bits = oracle.kc_update(k, wk, cos, sin, sl, b, 10)
    part, _ = oracle.kc_update(k, wk, cos, sin, sl, b, 10, block_begin=np.array([9, 2], dtype=np.int32),
                               block_end=np.array([10, 4], dtype=np.int32))
    np.testing.assert_array_equal(part[0, :, 9], full[0, :, 9])
    np.testing.assert_array_equal(part[1, :, 2:4], full[1, :, 2:4])
    assert np.isnan(part[0, :, :9]).all() and np.isnan(part[1, :, :2]).all() and np.isnan(part[1, :, 4:]).all()
    # same keys scattered into a paged pool
    npg = 10
    pool = torch.zeros(2 * npg + 1, 2, b, D, dtype=torch.bfloat16)
    pt = torch.zeros(2, npg, dtype=torch.int32)
    order = torch.randperm(2 * npg, generator=torch.Generator().manual_seed(1)) + 1
    for i in range(2):
        for p in range(npg):
            pg = int(order[i * npg + p]); pt[i, p] = pg
            pool[pg] = k[i, :, p * b:(p + 1) * b]
    paged, _ = oracle.kc_update(pool, wk, cos, sin, sl, b, 10, page_table=pt, page_size=b)
    np.testing.assert_array_equal(paged, full)


def test_rounding_to_bf16_is_nearest_even_without_double_rounding():
    # bf16 has 7 explicit mantissa bits (spacing 2^-7 at 1.0).  The rounding helper is internal to the
    # oracle, so it is exercised through the Q branch with d = Dg = 2, g = 1 at position 0:
    # y_0 = sum_c w[0][c] * x[c] builds values such as 1 + 2^-8 exactly from bf16-representable terms.
    def through_q(terms):
        """terms: list of (w, x) bf16-representable pairs; returns (fp64 sum, bf16 bits) of feature 0."""
        n = len(terms)
        d = max(2, n + (n % 2))
        q = torch.zeros(1, 1, d, dtype=torch.bfloat16); w = torch.zeros(1, 2, d, dtype=torch.bfloat16)
        for c, (a, b_) in enumerate(terms):
            w[0, 0, c] = a; q[0, 0, c] = b_
        cos = torch.ones(1, 1); sin = torch.zeros(1, 1)
        out, bits = oracle.gate_q(q, w, cos, sin, torch.tensor([1], dtype=torch.int32))
        return out[0, 0, 0], bits[0, 0, 0]
    cases = [
        ([(1.0, 1.0), (2.0 ** -8, 1.0)], 1.0),                       # tie -> even (1.0)
        ([(1.0, 1.0), (2.0 ** -8, 1.0), (2.0 ** -7, 1.0)], 1.0 + 2.0 ** -6),   # 1 + 3*2^-8: tie -> even (1 + 2^-6)
        ([(1.0, 1.0), (2.0 ** -8, 1.0), (2.0 ** -40, 1.0)], 1.0 + 2.0 ** -7),  # just above the tie
        ([(1.0, 1.0), (2.0 ** -8, 1.0), (-(2.0 ** -40), 1.0)], 1.0),           # just below the tie
        ([(-1.0, 1.0), (-(2.0 ** -8), 1.0)], -1.0),
        # double-rounding trap: 1 + 2^-8 + 2^-30 rounds to fp32 1 + 2^-8 (tie!) if rounded twice; correct is up
        ([(1.0, 1.0), (2.0 ** -8, 1.0), (2.0 ** -30, 1.0)], 1.0 + 2.0 ** -7),
    ]
    for terms, expect in cases:
        val, bits = through_q(terms)
        assert Fraction(val) == sum(Fraction(a) * Fraction(b_) for a, b_ in terms)
        got = torch.tensor([int(bits)], dtype=torch.int32).to(torch.int16).view(torch.bfloat16).double().item()
        assert got == expect, (terms, got, expect)
