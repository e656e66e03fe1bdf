"""Shared helpers of the GPU parity tests: run the fp64 oracle on copies of device tensors and
compare with the tolerances of the benchmark definition."""
import math

import numpy as np
import torch

import oracle
from oracle import KVLayout

# Tolerances.  Contract (benchmark definition): |out - ref| <= 1e-2 elementwise and
# max|out - ref| <= 1e-2 * max|ref| per row for bf16-in / fp32-accumulate outputs, lse within
# 1e-3.  The fp32-output runs are held to a much tighter bar, derived from the arithmetic: inputs are
# exact bf16, logits and outputs accumulate in fp32, and the MFMA kernel feeds the probabilities
# to the PV product as hi + lo bf16 pairs (2^-17 relative), so 2e-4 absolute / 4e-4 row-relative
# holds with margin and catches a dropped block or token that the 1e-2 contract would let through.
ATOL_BF16 = 1e-2
RTOL_ROW_BF16 = 1e-2
LSE_TOL = 1e-3
ATOL_F32 = 2e-4
RTOL_ROW_F32 = 4e-4
LSE_TOL_TIGHT = 1e-4


def cpu(t):
    if t is None or isinstance(t, np.ndarray):
        return t
    return t.detach().cpu()


def oracle_decode(inp, block_idx, nblk, group_filter=None):
    w = inp.w
    kv = KVLayout(cpu(inp.k), cpu(inp.v), cpu(inp.page_table), inp.page_size)
    return oracle.sparse_decode(cpu(inp.q), kv, inp.seqlens_cpu, cpu(block_idx), cpu(nblk), w.block_size,
                                w.scale, group_filter=group_filter)


def oracle_gate(inp, mode=oracle.SELECT_TOPK, threshold=0.0, max_sel=None, return_scores=False):
    w = inp.w
    return oracle.gate_select(cpu(inp.q_gate), cpu(inp.kc), inp.seqlens_cpu, w.block_size, mode=mode,
                              budget_tokens=w.budget_tokens, budget_blocks=cpu(inp.budget_blocks),
                              threshold=threshold, max_sel=max_sel or inp.max_sel, return_scores=return_scores)


def check_decode(out, lse, ref_out, ref_lse, *, tight, what=""):
    """Element-by-element comparison of a GPU result with the oracle's."""
    o = out.detach().float().cpu().numpy().astype(np.float64)
    l = lse.detach().cpu().numpy().astype(np.float64)
    sel = ~np.isnan(ref_lse)                       # rows the oracle computed
    assert sel.any(), "oracle computed nothing"
    atol, rtol, ltol = (ATOL_F32, RTOL_ROW_F32, LSE_TOL_TIGHT) if tight else (ATOL_BF16, RTOL_ROW_BF16, LSE_TOL)
    ro, rl = ref_out[sel], ref_lse[sel]
    go, gl = o[sel], l[sel]
    assert np.isfinite(go).all(), f"{what}: non-finite output"
    err = np.abs(go - ro)
    assert err.max() <= atol, f"{what}: max abs err {err.max():.3e} > {atol}"
    row_ref = np.abs(ro).max(axis=-1)
    row_err = err.max(axis=-1)
    nz = row_ref > 0
    if nz.any():
        rel = (row_err[nz] / row_ref[nz]).max()
        assert rel <= rtol, f"{what}: max row-relative err {rel:.3e} > {rtol}"
    assert (row_err[~nz] == 0).all(), f"{what}: empty rows must be exactly zero"
    inf = np.isneginf(rl)
    assert (np.isneginf(gl) == inf).all(), f"{what}: -inf lse pattern differs"
    if (~inf).any():
        le = np.abs(gl[~inf] - rl[~inf]).max()
        assert le <= ltol, f"{what}: max lse err {le:.3e} > {ltol}"
    return float(err.max())


def check_indices(block_idx, nblk, ref_idx, ref_cnt, what=""):
    gi = block_idx.detach().cpu().numpy()
    gc = nblk.detach().cpu().numpy()
    if not np.array_equal(gc, ref_cnt):
        bad = np.argwhere(gc != ref_cnt)
        raise AssertionError(f"{what}: nblk differs at {bad[:5].tolist()} (of {len(bad)})")
    if not np.array_equal(gi, ref_idx):
        bad = np.argwhere(gi != ref_idx)
        raise AssertionError(f"{what}: block_idx differs at {bad[:5].tolist()} (of {len(bad)})")


def pick_threshold(scores, seqlens, block_size, dg, target_keep):
    """A threshold at the midpoint between two adjacent softmax values (pooled over all groups)
    such that about `target_keep` of the full blocks are kept: the margin to the nearest
    probability is as large as it can be, so 1-ulp differences in exp cannot flip a decision."""
    probs = []
    B, Hkv, _ = scores.shape
    for i in range(B):
        nfull = int(seqlens[i]) // block_size
        if nfull == 0:
            continue
        x = scores[i, :, :nfull] / math.sqrt(dg)
        x = x - x.max(axis=1, keepdims=True)
        e = np.exp(x)
        probs.append((e / e.sum(axis=1, keepdims=True)).ravel())
    p = np.sort(np.concatenate(probs))
    cut = int(round((1.0 - target_keep) * len(p)))
    cut = min(max(cut, 1), len(p) - 1)
    # widen to the largest gap in a small neighbourhood
    lo, hi = max(1, cut - 8), min(len(p) - 1, cut + 8)
    gaps = p[lo:hi + 1] - p[lo - 1:hi]
    c = lo + int(np.argmax(gaps))
    return float(0.5 * (p[c - 1] + p[c]))


def oracle_decode_on_groups(inp, block_idx, nblk, groups, host_kv=None):
    """Oracle decode of a sample of (sequence, kv-head) groups of a large device-resident workload:
    only the sampled groups' K/V (or, for a paged cache, the sampled heads' pools) are copied to
    the host.  `host_kv` (a dict the caller keeps) caches the host copies of the page pools per kv
    head across calls on the same tensors.  Returns (out [n,g,d], lse [n,g]) in the order of
    `groups` (flat ids i*Hkv + h)."""
    w = inp.w
    g, d = w.g, w.d
    groups = np.asarray(groups)
    bi, hi = groups // w.Hkv, groups % w.Hkv
    tb = torch.as_tensor(bi)
    q_s = torch.stack([inp.q[int(b), int(h) * g:(int(h) + 1) * g] for b, h in zip(bi, hi)]).cpu()
    sl_s = inp.seqlens_cpu[tb].contiguous()
    idx_c, cnt_c = cpu(block_idx), cpu(nblk)
    if isinstance(idx_c, np.ndarray):
        idx_c, cnt_c = torch.as_tensor(idx_c), torch.as_tensor(cnt_c)
    idx_s = torch.stack([idx_c[int(b), int(h)] for b, h in zip(bi, hi)]).unsqueeze(1).contiguous()
    cnt_s = torch.stack([cnt_c[int(b), int(h)] for b, h in zip(bi, hi)]).unsqueeze(1).contiguous()
    n = len(groups)
    if inp.page_table is None:
        S_max = int(inp.seqlens_cpu.max())
        ks = torch.stack([inp.k[int(b), int(h), :S_max] for b, h in zip(bi, hi)]).unsqueeze(1).cpu()
        vs = torch.stack([inp.v[int(b), int(h), :S_max] for b, h in zip(bi, hi)]).unsqueeze(1).cpu()
        return oracle.sparse_decode(q_s, KVLayout(ks, vs), sl_s, idx_s, cnt_s, w.block_size, w.scale)
    out = np.zeros((n, g, d)); lse = np.zeros((n, g))
    pt_all = inp.page_table.cpu()
    for h in sorted(set(int(x) for x in hi)):
        m = np.nonzero(hi == h)[0]
        tm = torch.as_tensor(m)
        if host_kv is not None and h in host_kv:
            kh, vh = host_kv[h]
        else:
            kh, vh = inp.k[:, h:h + 1].cpu(), inp.v[:, h:h + 1].cpu()
            if host_kv is not None:
                host_kv[h] = (kh, vh)
        kv = KVLayout(kh, vh, pt_all[tb[tm]].contiguous(), inp.page_size)
        o, l = oracle.sparse_decode(q_s[tm], kv, sl_s[tm], idx_s[tm], cnt_s[tm], w.block_size, w.scale)
        out[m], lse[m] = o, l
    return out, lse


def gather_groups(t, w, groups, per_head):
    """Rows of a [B,Hq,...] (per_head=g) or [B,Hkv,...] (per_head=1) device tensor for sampled groups."""
    groups = np.asarray(groups)
    bi, hi = groups // w.Hkv, groups % w.Hkv
    return torch.stack([t[int(b), int(h) * per_head:(int(h) + 1) * per_head] for b, h in zip(bi, hi)])


def pick_top_p(scores, seqlens, block_size, dg, lo, hi, tries=64, seed=0):
    """A nucleus mass p in [lo, hi] that keeps every group's accumulated probability curve as far
    as possible from p at the cut (so the order of summation cannot move a cut)."""
    curves = []
    B, Hkv, _ = scores.shape
    for i in range(B):
        nfull = int(seqlens[i]) // block_size
        for h in range(Hkv):
            if nfull == 0:
                continue
            s = scores[i, h, :nfull]
            x = s / math.sqrt(dg)
            e = np.exp(x - x.max())
            P = e / e.sum()
            order = np.lexsort((np.arange(nfull), -s))
            curves.append(np.cumsum(P[order]))
    rng = np.random.default_rng(seed)
    best, best_margin = None, -1.0
    for p in rng.uniform(lo, hi, size=tries):
        margin = min(np.abs(c - p).min() for c in curves)
        if margin > best_margin:
            best, best_margin = float(p), margin
    assert best_margin > 1e-10, best_margin
    return best
