#!/usr/bin/env python3
"""Decode-attention benchmark of the SeerAttention-R hot path on one MI355X.

A step = one decode step of one attention layer for the whole batch: AttnGate block selection
(gate score + select) followed by the block-sparse flash-decode (split-K + LSE merge), all inputs
already resident in HBM.  value = tokens/s = batch / step time.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4] [--also c2,c3,c1,c5]

Besides the contract fields the line carries: the roofline of the dominant kernel (the split-K
decode kernel) and of the gate kernels from HIP events around every launch inside the timed steps
(mean, median and minimum), the speed-up over the library's own dense flash-decode, the fp64 CPU
oracle timed on a sample of the same workload (which doubles as a parity check that fails the run),
and compact entries for the other benchmark configurations: c2, c3 (paged, block 128), c1 (latency,
cold and warm) and the c5 sweep (top-k and threshold selection, block 64 and 128, 50-95 % sparsity).
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E peak
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix-core peak
CSRC = os.path.join(ROOT, "paper_2506_08889_amd", "csrc")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def kernel_sources_hash() -> str:
    """Fingerprint of the kernel sources: hardware-counter figures committed under profiles/ are only
    quoted while the kernels they were measured on are the ones in the tree."""
    h = hashlib.sha256()
    for name in sorted(os.listdir(CSRC)):
        if name.endswith((".hip", ".h")):
            with open(os.path.join(CSRC, name), "rb") as f:
                h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def committed_traffic(workload: str, key: str = "decode_bytes"):
    """Hardware-counter HBM bytes per launch (key "decode_bytes": split kernel plus merge kernel where one
    runs; "gate_bytes": score plus select kernel), or None when there is no committed measurement for
    this workload or it was taken on other kernel sources."""
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
            rec = json.load(f)
    except (OSError, ValueError):
        return None
    if rec.get("kernel_sources_sha256_16") != kernel_sources_hash():
        return None
    return rec.get(workload, {}).get(key)


def stats_us(ms_list):
    """mean / median / min of a list of durations in ms, as microseconds."""
    if not ms_list:
        return None
    us = [x * 1e3 for x in ms_list]
    return {"mean": statistics.fmean(us), "median": statistics.median(us), "min": min(us), "n": len(us)}


def algorithmic_bytes(w, bs, seqlens_cpu, nblk_cpu, idx_cpu, max_sel):
    """Bytes the method itself must move per step (decode and gate separately)."""
    import torch
    S = seqlens_cpu.to(torch.int64)
    nb = (S + bs - 1) // bs
    nfull = S // bs
    # valid tokens of the selected blocks: every selected block is full except a selected last partial one
    idx = idx_cpu.to(torch.int64)
    valid = (idx >= 0) & (idx < nb[:, None, None])
    tok = torch.where(valid, torch.minimum(torch.full_like(idx, bs), S[:, None, None] - idx * bs), torch.zeros_like(idx))
    sel_tokens = int(tok.sum())
    groups = w.B * w.Hkv
    kv_bytes = sel_tokens * 2 * w.d * 2
    n_entries = int(nblk_cpu.sum())
    decode = kv_bytes + 4 * n_entries + groups * (w.g * w.d * 2 * 2 + 4 * w.g)
    gate = int(nfull.sum()) * w.Hkv * w.Dg * 2 + groups * (w.Dg * 2 + 4) + 4 * n_entries
    dense_tokens = int(S.sum()) * w.Hkv
    dense = dense_tokens * 2 * w.d * 2 + groups * (w.g * w.d * 2 * 2 + 4 * w.g)
    return {"decode": decode, "gate": gate, "dense": dense, "selected_tokens": sel_tokens,
            "total_tokens": dense_tokens, "kv_bytes": kv_bytes}


class Bench:
    """Device-resident inputs of one workload plus the step functions that are timed."""

    def __init__(self, args, seer, synth, torch, w, projected_gate=False):
        self.args, self.seer, self.synth, self.torch, self.w = args, seer, synth, torch, w
        dev = self.dev = "cuda:0"
        seer.set_knob(0, args.impl)
        seer.set_knob(1, args.splits)
        seer.set_knob(3, args.gate_impl)
        t0 = time.time()
        base = self.base = synth.make_inputs(w, dev)
        self.bs = w.block_size
        full_kv_bytes = base.k.numel() * 2 * 2
        # several KV caches (small workloads) and several query sets are cycled so that no step finds its
        # K/V rows in the 256 MB memory-side cache or the L2s
        self.kv_copies = args.kv_copies or (1 if full_kv_bytes > (8 << 30) else max(1, min(4, (8 << 30) // max(full_kv_bytes, 1))))
        self.caches = [(base.k, base.v)]
        gen = synth.generator(dev, w.seed + 1000)
        for _ in range(self.kv_copies - 1):
            self.caches.append((synth.randn_bf16(tuple(base.k.shape), dev, gen), synth.randn_bf16(tuple(base.v.shape), dev, gen)))
        self.R = R = max(1, args.rotate)
        self.qs, self.qgs = [base.q], [base.q_gate]
        for _ in range(R - 1):
            self.qs.append(synth.randn_bf16(tuple(base.q.shape), dev, gen))
            self.qgs.append(synth.randn_bf16(tuple(base.q_gate.shape), dev, gen))
        self.kc = base.kc
        if projected_gate:
            # gate inputs through the AttnGate projections (Eq. 1a / 1b) with random weights, off the clock:
            # the K cache stands in for the pre-RoPE keys, the queries for the pre-RoPE queries
            gen2 = synth.generator(dev, w.seed + 2000)
            wq, wk = synth.gate_weights(w, dev, gen2)
            rcos, rsin = synth.rope_tables(base.nb_max * self.bs + 1, w.Dg, device=dev)
            self.kc = torch.zeros_like(base.kc)
            seer.kc_update(base.k, wk, rcos, rsin, base.seqlens, self.bs, self.kc, page_table=base.page_table,
                           page_size=base.page_size)
            self.qgs = [seer.gate_q(q, wq, rcos, rsin, base.seqlens) for q in self.qs]
            del wq, wk, rcos, rsin
        torch.cuda.synchronize()
        B, Hq, Hkv, d = w.B, w.Hq, w.Hkv, w.d
        self.out = torch.empty(B, Hq, d, dtype=torch.bfloat16, device=dev)
        self.lse = torch.empty(B, Hq, dtype=torch.float32, device=dev)
        self.ws_gate = torch.empty(seer.gate_workspace_bytes(B, Hkv, base.nb_max), dtype=torch.uint8, device=dev)
        self.ws_dense = None
        self.configure(seer.SELECT_TOPK, base.max_sel, base.budget_blocks, 0.0)
        log(f"[bench] {w.name}: B={B} Hq={Hq} Hkv={Hkv} bs={self.bs} paged={w.paged}; inputs in {time.time() - t0:.1f}s; "
            f"kv copies {self.kv_copies}, query sets {R}, KV cache {full_kv_bytes / 2**30:.2f} GiB")

    def configure(self, mode, max_sel, budget_blocks, threshold):
        """Selection mode of the following steps (allocates the index lists and the decode workspace)."""
        torch, seer, w = self.torch, self.seer, self.w
        self.mode, self.max_sel, self.budget_blocks, self.threshold = mode, max_sel, budget_blocks, threshold
        # lists of very different lengths: mixed sequence lengths, per-sequence budgets, threshold selection
        self.ragged = w.seqlen_dist != "fixed" or w.budget_tokens == 0 or mode != seer.SELECT_TOPK
        self.idxs = [torch.empty(w.B, w.Hkv, max_sel, dtype=torch.int32, device=self.dev) for _ in range(self.R)]
        self.cnts = [torch.empty(w.B, w.Hkv, dtype=torch.int32, device=self.dev) for _ in range(self.R)]
        self.ws_dec = torch.empty(seer.decode_workspace_bytes(w.B, w.Hq, w.Hkv, w.d, max_sel), dtype=torch.uint8, device=self.dev)

    def gate(self, r):
        w = self.w
        self.seer.gate_select(self.qgs[r], self.kc, self.base.seqlens, self.bs, mode=self.mode,
                              budget_tokens=w.budget_tokens, budget_blocks=self.budget_blocks, threshold=self.threshold,
                              max_sel=self.max_sel, block_idx=self.idxs[r], nblk=self.cnts[r], workspace=self.ws_gate,
                              ragged=self.ragged)

    def decode(self, r, cache):
        k, v = self.caches[cache]
        self.seer.sparse_decode(self.qs[r], k, v, self.base.seqlens, self.idxs[r], self.cnts[r], self.bs, self.w.scale,
                                page_table=self.base.page_table, page_size=self.base.page_size, out=self.out,
                                lse=self.lse, workspace=self.ws_dec, ragged=self.ragged)

    def step(self, i):
        self.gate(i % self.R)
        self.decode(i % self.R, i % self.kv_copies)

    def dense_step(self, i):
        w, base = self.w, self.base
        if self.ws_dense is None:
            self.ws_dense = self.torch.empty(self.seer.decode_workspace_bytes(w.B, w.Hq, w.Hkv, w.d, base.nb_max),
                                             dtype=self.torch.uint8, device=self.dev)
        k, v = self.caches[i % self.kv_copies]
        self.seer.dense_decode(self.qs[i % self.R], k, v, base.seqlens, base.nb_max, self.bs, w.scale,
                               page_table=base.page_table, page_size=base.page_size, out=self.out, lse=self.lse,
                               workspace=self.ws_dense, ragged=w.seqlen_dist != "fixed")

    # ---- timing -----------------------------------------------------------------------------------
    def timed(self, fn, n, start=0):
        """Mean wall-clock ms per call of n back-to-back calls, bracketed by synchronisations."""
        torch = self.torch
        torch.cuda.synchronize()
        t = time.perf_counter()
        for i in range(n):
            fn(start + i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3 / n

    def profiled(self, fn, n, start=0, classes=(0, 1, 2, 3)):
        """The same calls with HIP events around every kernel launch (recorded by the library on the stream
        the kernels run on) and around every call: per-kernel and per-call mean / median / min in us."""
        torch, seer = self.torch, self.seer
        seer.profile_reset()
        seer.profile_enable(True)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        torch.cuda.synchronize()
        for i in range(n):
            ev[i][0].record()
            fn(start + i)
            ev[i][1].record()
        torch.cuda.synchronize()
        seer.profile_enable(False)
        kern = {seer.KERNEL_CLASSES[c]: stats_us(seer.profile_durations(c)) for c in classes}
        seer.profile_reset()
        return kern, stats_us([a.elapsed_time(b) for a, b in ev])

    def selection(self):
        """Byte model from the selection the gate actually makes for query set 0."""
        torch = self.torch
        self.gate(0)
        self.decode(0, 0)
        torch.cuda.synchronize()
        idx_cpu, cnt_cpu = self.idxs[0].cpu(), self.cnts[0].cpu()
        ab = algorithmic_bytes(self.w, self.bs, self.base.seqlens_cpu, cnt_cpu, idx_cpu, self.max_sel)
        ab["sparsity"] = 1.0 - ab["selected_tokens"] / max(ab["total_tokens"], 1)
        return ab, idx_cpu, cnt_cpu

    def measure(self, steps, warmup, dense_steps):
        """Timed region + per-kernel pass + dense baseline -> the figures every workload reports."""
        for i in range(warmup):
            self.step(i)
        ms_step = self.timed(self.step, steps, warmup)
        kern, step_ev = self.profiled(self.step, steps, warmup)
        ab, idx_cpu, cnt_cpu = self.selection()
        # the decode call alone (split + merge launches), queued back to back on lists made beforehand: no
        # event records between the kernels, which add 1-3 us to each short kernel's HIP-event figure
        for r in range(self.R):
            self.gate(r)
        dec_b2b_us = self.timed(lambda i: self.decode(i % self.R, i % self.kv_copies), steps, warmup) * 1e3
        split, merge = kern["decode_split"], kern["decode_merge"]
        merge_mean = merge["mean"] if merge else 0.0
        dec_us = split["mean"] + merge_mean
        gate_us = (kern["gate_score"]["mean"] if kern["gate_score"] else 0.0) + kern["gate_select"]["mean"]
        achieved = ab["decode"] / (dec_us * 1e-6) / 1e9
        res = {
            "ms_per_step": ms_step,
            "step_us": {"launch_inclusive_mean": ms_step * 1e3, "gpu_events": step_ev,
                        "kernels_only_mean": sum(v["mean"] for v in kern.values() if v)},
            "kernels_us": kern,
            "realised_sparsity": ab["sparsity"],
            # (token, kv head) pairs of the selected blocks read per second of the whole step
            "selected_kv_tokens_per_s": ab["selected_tokens"] / (ms_step * 1e-3),
            "roofline": {"bound": "hbm",
                         "kernel": "seer_decode_split (sparse)" + (" + seer_decode_merge" if merge else ""),
                         "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                         "traffic": committed_traffic(self.w.name) if self.mode == self.seer.SELECT_TOPK else None,
                         "algorithmic_bytes_per_launch": ab["decode"], "avg_kernel_us": dec_us,
                         "split_kernel_us": split, "merge_kernel_us": merge,
                         "frac_split_kernel_alone": ab["decode"] / (split["mean"] * 1e-6) / 1e9 / HBM_PEAK_GBPS,
                         "frac_at_min_duration": ab["decode"] / ((split["min"] + (merge["min"] if merge else 0.0)) * 1e-6) / 1e9 / HBM_PEAK_GBPS,
                         "decode_call_us_back_to_back": dec_b2b_us,
                         "frac_decode_calls_back_to_back": ab["decode"] / (dec_b2b_us * 1e-6) / 1e9 / HBM_PEAK_GBPS},
            "gate_roofline": {"bound": "hbm", "kernel": "seer_gate_score + seer_gate_select" if kern["gate_score"] else "seer_gate_select (fused: scores and selection)",
                              "achieved": ab["gate"] / (gate_us * 1e-6) / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                              "frac": ab["gate"] / (gate_us * 1e-6) / 1e9 / HBM_PEAK_GBPS,
                              "traffic": committed_traffic(self.w.name, "gate_bytes") if self.mode == self.seer.SELECT_TOPK else None,
                              "algorithmic_bytes_per_launch": ab["gate"], "avg_kernel_us": gate_us},
        }
        if dense_steps > 0:
            for i in range(2):
                self.dense_step(i)
            ms_dense = self.timed(self.dense_step, dense_steps)
            dk, _ = self.profiled(self.dense_step, dense_steps, classes=(2, 3))
            d_us = dk["decode_split"]["mean"] + (dk["decode_merge"]["mean"] if dk["decode_merge"] else 0.0)
            dense_gbps = ab["dense"] / (d_us * 1e-6) / 1e9
            res["dense"] = {"ms_per_step": ms_dense, "kernel_us": d_us, "GBps": dense_gbps,
                            "pct_hbm_peak": 100.0 * dense_gbps / HBM_PEAK_GBPS}
            res["speedup_vs_dense"] = {"decode_only": d_us / dec_us, "with_gate": ms_dense / ms_step,
                                       "ideal": 1.0 / max(1.0 - ab["sparsity"], 1e-9)}
        return res, ab, idx_cpu, cnt_cpu

    def describe(self):
        w, base = self.w, self.base
        return (f"{w.name}: batch {w.B}, {w.Hq} q / {w.Hkv} kv heads, head_dim {w.d}, block {self.bs}, "
                f"seqlen {int(base.seqlens_cpu.min())}..{int(base.seqlens_cpu.max())}, max_sel {self.max_sel}, "
                f"{'paged' if w.paged else 'contiguous'} KV")

    def release(self):
        self.caches = self.base = self.qs = self.qgs = self.kc = self.ws_dec = self.ws_dense = self.ws_gate = None
        self.idxs = self.cnts = None
        self.torch.cuda.empty_cache()


def main_workload(args, seer, synth, torch, np):
    """The headline workload with every leg: step, kernels, dense baseline, stream-read ceiling, front-end,
    multi-token decode, training forward, CPU oracle."""
    w = synth.CONFIGS[args.workload]
    b = Bench(args, seer, synth, torch, w, projected_gate=(w.name == "c5"))
    dev, base, bs = b.dev, b.base, b.bs
    B, Hq, Hkv, d = w.B, w.Hq, w.Hkv, w.d
    res, ab, idx_cpu, cnt_cpu = b.measure(args.steps, args.warmup, args.dense_steps)
    log(f"[bench] {w.name}: step {res['ms_per_step'] * 1e3:.1f} us; kernels " +
        ", ".join(f"{k}={v['mean']:.1f}" for k, v in res["kernels_us"].items() if v))

    # ---- plain streaming read of the K cache: the practical HBM ceiling on this machine
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    probe_src = b.caches[0][0].view(-1)[: min(b.caches[0][0].numel(), 4 << 30)]     # <= 8 GiB
    for _ in range(2):
        seer.hbm_read_probe(probe_src, sink)
    pk, _ = b.profiled(lambda i: seer.hbm_read_probe(probe_src, sink), 5, classes=(4,))
    stream_gbps = probe_src.numel() * 2 / (pk["stream_read"]["mean"] * 1e-6) / 1e9

    # ---- AttnGate front-end (reported beside the step, not part of `value`): the per-step query
    # branch, the K Compression Cache rebuilt for every block (as after a prefill; the K tensor stands in
    # for the pre-RoPE keys) and the one-block update a sequence needs when it completes a block.
    gen2 = synth.generator(dev, w.seed + 2000)
    wq, wk = synth.gate_weights(w, dev, gen2)
    rcos, rsin = synth.rope_tables(base.nb_max * bs + 1, w.Dg, device=dev)
    kc_out = torch.empty_like(base.kc)
    qg_out = torch.empty_like(base.q_gate)
    nfull_cpu = (base.seqlens_cpu // bs).to(torch.int32)
    last_begin = (nfull_cpu - 1).clamp(min=0).to(dev)
    last_end = nfull_cpu.to(dev)

    def fe_q(i):
        seer.gate_q(b.qs[i % b.R], wq, rcos, rsin, base.seqlens, q_gate=qg_out)

    def fe_full(i):
        seer.kc_update(b.caches[0][0], wk, rcos, rsin, base.seqlens, bs, kc_out, page_table=base.page_table,
                       page_size=base.page_size)

    def fe_last(i):
        seer.kc_update(b.caches[0][0], wk, rcos, rsin, base.seqlens, bs, kc_out, max_blocks=1,
                       block_begin=last_begin, block_end=last_end, page_table=base.page_table, page_size=base.page_size)

    def step_from_raw_q(i):      # the decode step with the gate query made from the raw queries inside the gate call
        r = i % b.R
        seer.gate_select_q(b.qs[r], wq, rcos, rsin, b.kc, base.seqlens, bs, mode=b.mode, budget_tokens=w.budget_tokens,
                           budget_blocks=b.budget_blocks, threshold=b.threshold, max_sel=b.max_sel, block_idx=b.idxs[r],
                           nblk=b.cnts[r], workspace=b.ws_gate, ragged=b.ragged)
        b.decode(r, i % b.kv_copies)

    for fn in (fe_q, fe_full, fe_last, step_from_raw_q):
        fn(0)
    ms_step_q = b.timed(step_from_raw_q, args.steps, args.warmup)
    ms_q = b.timed(fe_q, 20)
    kq, _ = b.profiled(fe_q, 20, classes=(5,))
    kf, _ = b.profiled(fe_full, 3, classes=(6,))
    kl, _ = b.profiled(fe_last, 20, classes=(6,))
    kc_bytes = int(nfull_cpu.to(torch.int64).sum()) * Hkv * (bs * w.d * 2 + w.Dg * 2)
    full_us = kf["kc_update"]["mean"]
    frontend = {"gate_q_us": kq["gate_q"], "gate_q_ms_per_call": ms_q,
                "kc_update_all_blocks": {"kernel_us": full_us, "algorithmic_bytes": kc_bytes,
                                         "GBps": kc_bytes / (full_us * 1e-6) / 1e9,
                                         "frac_hbm_peak": kc_bytes / (full_us * 1e-6) / 1e9 / HBM_PEAK_GBPS},
                "kc_update_last_block_us": kl["kc_update"],
                "ms_per_step_from_raw_q": ms_step_q,
                "q_branch_cost_per_step_us": (ms_step_q - res["ms_per_step"]) * 1e3}
    del wq, wk, rcos, rsin, kc_out

    # ---- several new tokens per call (multi-token / speculative decoding): same bytes, q_len x the tokens
    multi = None
    if 16 // w.g >= 2 and bs % 32 == 0 and args.impl != 1:      # the matrix-core kernel only
        T = min(16 // w.g, 4)
        qm = synth.randn_bf16((B, T, Hq, d), dev, synth.generator(dev, w.seed + 3000))
        out_m = torch.empty(B, T, Hq, d, dtype=torch.bfloat16, device=dev)
        lse_m = torch.empty(B, T, Hq, dtype=torch.float32, device=dev)
        ws_m = torch.empty(seer.decode_workspace_bytes(B, Hq * T, Hkv, d, b.max_sel), dtype=torch.uint8, device=dev)

        def mt(i):
            k_, v_ = b.caches[i % b.kv_copies]
            seer.sparse_decode_multi(qm, k_, v_, base.seqlens, b.idxs[i % b.R], b.cnts[i % b.R], bs, w.scale,
                                     page_table=base.page_table, page_size=base.page_size, out=out_m, lse=lse_m,
                                     workspace=ws_m, ragged=b.ragged)

        for i in range(3):
            mt(i)
        ms_mt = b.timed(mt, 10)
        km, _ = b.profiled(mt, 10, classes=(2,))
        multi = {"q_len": T, "query_rows_per_kv_head": T * w.g, "split_kernel_us": km["decode_split"], "ms_per_call": ms_mt,
                 "decode_tokens_per_s": B * T / (ms_mt * 1e-3)}
        del qm, out_m, lse_m, ws_m

    # ---- training-side forward: causal attention + gate ground truth over one whole sequence
    train = None
    if args.train_tokens > 0 and bs % 32 == 0:
        Tt = args.train_tokens
        gen_t = synth.generator(dev, w.seed + 4000)
        q_t = synth.randn_bf16((1, Tt, Hq, d), dev, gen_t)
        k_t = synth.randn_bf16((1, Hkv, Tt, d), dev, gen_t)
        v_t = synth.randn_bf16((1, Hkv, Tt, d), dev, gen_t)
        nb_t = (Tt + bs - 1) // bs
        out_t = torch.empty(1, Tt, Hq, d, dtype=torch.bfloat16, device=dev)
        lse_t = torch.empty(1, Tt, Hq, dtype=torch.float32, device=dev)
        gt_t = torch.empty(1, Hkv, Tt, nb_t, dtype=torch.float32, device=dev)
        ws_t = torch.empty(seer.attn_ground_truth_workspace_bytes(1, Tt, Hq, Hkv, d, bs), dtype=torch.uint8, device=dev)

        def tr(i):
            seer.attn_ground_truth(q_t, k_t, v_t, bs, w.scale, out=out_t, lse=lse_t, gt=gt_t, workspace=ws_t)

        for i in range(2):
            tr(i)
        ms_tr = b.timed(tr, 5)
        kt, _ = b.profiled(tr, 5, classes=(7, 8))
        flops = 4.0 * Hq * d * (Tt * (Tt + 1) / 2)          # QK^T and PV over the causal triangle
        fwd_ms = kt["attn_fwd"]["mean"] * 1e-3
        tf = flops / (fwd_ms * 1e-3) / 1e12
        train = {"workload": f"1 sequence of {Tt} tokens, {Hq} q / {Hkv} kv heads, block {bs}",
                 "ms_per_call": ms_tr, "attn_fwd_kernel_us": kt["attn_fwd"], "gt_finalize_kernel_us": kt["gt_finalize"],
                 "causal_flops": flops,
                 "roofline": {"bound": "mfma", "kernel": "seer_attn_fwd", "achieved": tf, "peak": MFMA_BF16_PEAK_TFLOPS,
                              "unit": "TFLOP/s", "frac": tf / MFMA_BF16_PEAK_TFLOPS, "traffic": None}}
        del q_t, k_t, v_t, out_t, lse_t, gt_t, ws_t

    if args.calibrate_copy_mib > 0:
        a = torch.empty(args.calibrate_copy_mib << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        b_ = torch.empty_like(a)
        for _ in range(3):
            b_.copy_(a)
        torch.cuda.synchronize()
        del a, b_

    roof = res["roofline"]
    result = {
        "metric": "sparse decode attention tokens/s + achieved HBM GB/s (% peak) at 90% sparsity",
        "value": B / (res["ms_per_step"] * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": b.describe(),
                   "step": "gate score + top-k select + sparse split-K decode + LSE merge",
                   "realised_sparsity": res["realised_sparsity"], "query_sets": b.R, "kv_copies": b.kv_copies,
                   "decode_impl": {0: "auto(mfma)", 1: "valu", 2: "mfma"}[args.impl], "ragged_lists_hint": b.ragged},
        "roofline": roof,
        "gate_roofline": res["gate_roofline"],
        "hbm_GBps_selected_kv": roof["achieved"], "pct_hbm_peak": 100.0 * roof["frac"],
        "selected_kv_tokens_per_s": res["selected_kv_tokens_per_s"],
        "step_us": res["step_us"],
        "kernels_us": res["kernels_us"],
        "stream_read_GBps": stream_gbps,
        "frontend": frontend,
        "multi_token_decode": multi,
        "training_forward": train,
        "dense": res.get("dense"), "speedup_vs_dense": res.get("speedup_vs_dense"),
        "paper_context": "the paper measures about 9x over FlashAttention-3 at 90% sparsity on H100 (other hardware: context, not a target)",
    }

    # ---- CPU oracle on a bounded sample of the same workload: the reported baseline, and a parity check
    # on the bench's own launch configuration that fails the run when it does not hold
    if not args.no_cpu_baseline:
        result.update(cpu_baseline_and_parity(args, b, idx_cpu, np, torch))
    b.release()
    return result


def cpu_baseline_and_parity(args, b, idx_cpu, np, torch):
    import oracle
    from oracle import KVLayout
    w, base, bs = b.w, b.base, b.bs
    B, Hkv, g, d = w.B, w.Hkv, w.g, w.d
    G = B * Hkv
    ns = min(args.cpu_sample, G)
    rng = np.random.default_rng(w.seed)
    groups = np.sort(rng.choice(G, size=ns, replace=False))
    bi, hi = groups // Hkv, groups % Hkv
    k0, v0 = b.caches[0]
    t0 = time.time()
    if base.page_table is None:
        S_max = int(base.seqlens_cpu.max())
        ks = torch.stack([k0[int(b_), int(h_), :S_max] for b_, h_ in zip(bi, hi)]).unsqueeze(1).cpu()
        vs = torch.stack([v0[int(b_), int(h_), :S_max] for b_, h_ in zip(bi, hi)]).unsqueeze(1).cpu()
        kvs = KVLayout(ks, vs)
    else:
        # a paged pool is copied once per distinct sampled kv head
        heads = sorted(set(int(h_) for h_ in hi))
        pools = {h_: (k0[:, h_:h_ + 1].cpu(), v0[:, h_:h_ + 1].cpu()) for h_ in heads}
        kvs = None
    qs_s = torch.stack([b.qs[0][int(b_), int(h_) * g:(int(h_) + 1) * g] for b_, h_ in zip(bi, hi)]).cpu()
    qg_s = torch.stack([b.qgs[0][int(b_), int(h_)] for b_, h_ in zip(bi, hi)]).unsqueeze(1).cpu()
    kc_s = torch.stack([b.kc[int(b_), int(h_)] for b_, h_ in zip(bi, hi)]).unsqueeze(1).cpu()
    sl_s = base.seqlens_cpu[torch.as_tensor(bi)].contiguous()
    bb_s = base.budget_blocks_cpu[torch.as_tensor(bi)].contiguous() if base.budget_blocks_cpu is not None else None
    log(f"[bench] sample of {ns} groups staged on the host in {time.time() - t0:.1f}s")
    t_cpu = None
    for _rep in range(3):      # best of three runs of the same sample
        t1 = time.perf_counter()
        oi, oc = oracle.gate_select(qg_s, kc_s, sl_s, bs, budget_tokens=w.budget_tokens, budget_blocks=bb_s, max_sel=b.max_sel)
        if kvs is not None:
            oo, ol = oracle.sparse_decode(qs_s, kvs, sl_s, oi, oc, bs, w.scale)
        else:
            oo = np.zeros((ns, g, d)); ol = np.zeros((ns, g))
            for h_ in heads:
                m = np.nonzero(hi == h_)[0]
                pt = base.page_table.cpu()[torch.as_tensor(bi[m])].contiguous()
                o_, l_ = oracle.sparse_decode(qs_s[m], KVLayout(pools[h_][0], pools[h_][1], pt, base.page_size),
                                              sl_s[m], oi[m], oc[m], bs, w.scale)
                oo[m], ol[m] = o_, l_
        t_rep = time.perf_counter() - t1
        t_cpu = t_rep if t_cpu is None else min(t_cpu, t_rep)
    est_step_s = t_cpu * G / ns
    b.gate(0)                  # the step the oracle just computed, once more (later legs reused the output buffers)
    b.decode(0, 0)
    torch.cuda.synchronize()
    idx_cpu = b.idxs[0].cpu()
    gi = idx_cpu.numpy().reshape(G, b.max_sel)[groups]
    go = b.out.float().cpu().numpy().reshape(B, Hkv, g, d)[bi, hi]
    gl = b.lse.cpu().numpy().reshape(B, Hkv, g)[bi, hi]
    err = np.abs(go - oo)
    row_ref = np.maximum(np.abs(oo).max(-1), 1e-30)
    fin = np.isfinite(ol)
    parity = {"groups": int(ns), "indices_bit_exact": bool(np.array_equal(gi, oi.reshape(ns, b.max_sel))),
              "max_abs_err_out_bf16": float(err.max()),
              "max_row_rel_err_out_bf16": float((err.max(-1) / row_ref).max()),
              "max_abs_err_lse": float(np.abs(gl[fin] - ol[fin]).max()) if fin.any() else 0.0}
    parity["ok"] = bool(parity["indices_bit_exact"] and parity["max_abs_err_out_bf16"] <= 1e-2 and
                        parity["max_row_rel_err_out_bf16"] <= 1e-2 and parity["max_abs_err_lse"] <= 1e-3 and
                        np.array_equal(np.isfinite(gl), fin))
    return {"cpu_baseline": {"value": B / est_step_s, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
                             "sample": f"{ns} of {G} (batch, kv-head) groups of the same workload, gate + decode, "
                                       f"best of 3 runs, {t_cpu:.2f} s of oracle time scaled by {G}/{ns}",
                             "oracle_step_s_estimate": est_step_s},
            "parity_on_sample": parity}


def compact(res, b):
    r = res["roofline"]
    out = {"workload": b.describe(), "value": b.w.B / (res["ms_per_step"] * 1e-3), "unit": "tokens/s",
           "ms_per_step": res["ms_per_step"], "step_us_gpu_events": res["step_us"]["gpu_events"],
           "realised_sparsity": res["realised_sparsity"], "selected_kv_tokens_per_s": res["selected_kv_tokens_per_s"],
           "ragged_lists_hint": b.ragged,
           "roofline": {k: r[k] for k in ("bound", "kernel", "achieved", "peak", "unit", "frac", "traffic",
                                          "algorithmic_bytes_per_launch", "avg_kernel_us", "frac_split_kernel_alone",
                                          "decode_call_us_back_to_back", "frac_decode_calls_back_to_back")},
           "gate_frac_hbm_peak": res["gate_roofline"]["frac"],
           "kernels_us": {k: ({"mean": v["mean"], "median": v["median"], "min": v["min"]} if v else None)
                          for k, v in res["kernels_us"].items()}}
    if "dense" in res:
        out["dense"] = res["dense"]
        out["speedup_vs_dense"] = res["speedup_vs_dense"]
    return out


def also_workload(args, name, seer, synth, torch):
    b = Bench(args, seer, synth, torch, synth.CONFIGS[name])
    res, _, _, _ = b.measure(args.steps, args.warmup, min(args.dense_steps, 3))
    out = compact(res, b)
    log(f"[bench] {name}: step {res['ms_per_step'] * 1e3:.1f} us, decode frac {out['roofline']['frac']:.3f}")
    b.release()
    return out


def graph_replay_us(b, torch, n):
    """One step (query set 0, cache 0) captured into a HIP graph on a stream of its own and replayed n
    times back to back: what a serving loop that replays its decode step pays per step, in us.  The
    library records no memset and allocates nothing, so the capture holds only its kernels."""
    s = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        b.step(0)                                   # warm-up on the capture stream
        s.synchronize()
        with torch.cuda.graph(g, stream=s):
            b.step(0)
    torch.cuda.synchronize()
    for _ in range(5):
        g.replay()
    torch.cuda.synchronize()
    t = time.perf_counter()
    for _ in range(n):
        g.replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t) * 1e6 / n


def c1_latency(args, seer, synth, torch):
    """The tiny configuration is latency-bound (1 MiB of selected KV): microseconds per step, once with
    128 KV caches cycled (cold: 512 MiB between re-uses, beyond the memory-side cache and the L2s) and once
    on one cache (warm).  No roofline claim."""
    import copy
    out = {"note": "latency-bound; no roofline claim"}
    for label, copies in (("cold_rotated", 128), ("warm", 1)):
        a = copy.copy(args)
        a.kv_copies = copies
        b = Bench(a, seer, synth, torch, synth.CONFIGS["c1"])
        for i in range(10):
            b.step(i)
        n = max(args.steps, 256 if copies > 1 else 50)
        ms = b.timed(b.step, n, 10)
        kern, ev = b.profiled(b.step, n, 10)
        out[label] = {"step_us_launch_inclusive_mean": ms * 1e3, "step_us_gpu_events": ev,
                      "kernels_us": {k: ({"mean": v["mean"], "median": v["median"], "min": v["min"]} if v else None)
                                     for k, v in kern.items()}}
        if copies == 1:
            out[label]["step_us_graph_replay_mean"] = graph_replay_us(b, torch, n)
        out["workload"] = b.describe()
        b.release()
    log(f"[bench] c1: cold {out['cold_rotated']['step_us_launch_inclusive_mean']:.1f} us, warm {out['warm']['step_us_launch_inclusive_mean']:.1f} us, "
        f"warm under graph replay {out['warm']['step_us_graph_replay_mean']:.1f} us")
    return out


def c5_sweep(args, seer, synth, torch, block_sizes, keeps):
    """End-to-end gate + decode on the batch-128 mixed-length paged configuration: token-budget and
    threshold selection at several sparsity levels, gate inputs through the AttnGate projections.  The
    threshold of a point is found by bisection on the library's own threshold selection so that it keeps
    about as many blocks as the token-budget run of the same point."""
    points = []
    for bs in block_sizes:
        w = synth.scaled(synth.CONFIGS["c5"], block_size=bs)
        b = Bench(args, seer, synth, torch, w, projected_gate=True)
        base = b.base
        for i in range(2):
            b.dense_step(i)
        dk, _ = b.profiled(b.dense_step, 3, classes=(2, 3))
        dense_us = dk["decode_split"]["mean"] + (dk["decode_merge"]["mean"] if dk["decode_merge"] else 0.0)
        ms_dense = b.timed(b.dense_step, 3)
        for keep in keeps:
            bb_cpu = synth.block_budgets(base.seqlens_cpu, bs, keep)
            b.configure(seer.SELECT_TOPK, int(bb_cpu.max()), bb_cpu.to(b.dev), 0.0)
            res, ab, _, cnt_cpu = b.measure(args.sweep_steps, 3, 0)
            target_blocks = int(cnt_cpu.sum())
            points.append(sweep_point("top-k", bs, keep, res, dense_us, ms_dense))
            # threshold mode: bisect tau (log scale) on the selection the library itself makes
            b.configure(seer.SELECT_THRESHOLD, base.nb_max, None, 0.0)
            lo, hi = 1e-9, 1.0
            for _ in range(40):
                b.threshold = (lo * hi) ** 0.5
                b.gate(0)
                if int(b.cnts[0].sum().item()) > target_blocks:
                    lo = b.threshold
                else:
                    hi = b.threshold
            b.threshold = hi
            res, ab, _, _ = b.measure(args.sweep_steps, 3, 0)
            pt = sweep_point("threshold", bs, keep, res, dense_us, ms_dense)
            pt["threshold"] = b.threshold
            points.append(pt)
            log(f"[bench] c5 b={bs} keep={keep}: top-k {points[-2]['step_us']:.0f} us ({points[-2]['decode_frac_hbm_peak']:.3f}), "
                f"threshold {pt['step_us']:.0f} us ({pt['decode_frac_hbm_peak']:.3f})")
        b.release()
    return points


def sweep_point(mode, bs, keep, res, dense_us, ms_dense):
    k = res["kernels_us"]
    return {"mode": mode, "block_size": bs, "target_sparsity": 1.0 - keep, "realised_sparsity": res["realised_sparsity"],
            "step_us": res["ms_per_step"] * 1e3, "step_us_median_gpu_events": res["step_us"]["gpu_events"]["median"],
            "gate_us": (k["gate_score"]["mean"] if k["gate_score"] else 0.0) + k["gate_select"]["mean"],
            "decode_split_us": k["decode_split"]["mean"], "decode_merge_us": k["decode_merge"]["mean"] if k["decode_merge"] else 0.0,
            "decode_frac_hbm_peak": res["roofline"]["frac"],
            "speedup_vs_dense_decode_only": dense_us / res["roofline"]["avg_kernel_us"],
            "speedup_vs_dense_with_gate": ms_dense / res["ms_per_step"],
            "ideal_speedup": 1.0 / max(1.0 - res["realised_sparsity"], 1e-9)}


def paper_sweep(args, seer, synth, torch):
    """Kernel speed-up sweep in the shape of the paper's kernel evaluation (Sec. 4.4): random tensors, 64
    query / 8 kv heads, head dim 128, block 64; sequence length 8k..128k, batch 1..16, block sparsity 0.5 /
    0.75 / 0.9 (uniformly random block lists, the same count for every group).  For every point the
    block-sparse decode (split kernel + merge) and the dense flash-decode of this library are timed with
    HIP events around every launch; prints a markdown table instead of the JSON line."""
    dev = "cuda:0"
    Hq, Hkv, d, bs = 64, 8, 128, 64
    scale = 1.0 / d ** 0.5
    gen = synth.generator(dev, 7)
    gcpu = torch.Generator().manual_seed(7)
    for k in (0, 1, 3):
        seer.set_knob(k, 0)

    def kernel_us(fn, n):
        for i in range(3):
            fn(i)
        seer.profile_reset()
        seer.profile_enable(True)
        for i in range(n):
            fn(i)
        torch.cuda.synchronize()
        seer.profile_enable(False)
        split, merge = seer.profile_durations(2), seer.profile_durations(3)
        seer.profile_reset()
        return (statistics.fmean(split) + (statistics.fmean(merge) if merge else 0.0)) * 1e3

    print("| seqlen | batch | sparsity | selected blocks | dense us | dense GB/s | sparse us | sparse GB/s | speed-up | ideal |")
    print("|---|---|---|---|---|---|---|---|---|---|")
    for S in (8192, 16384, 32768, 65536, 131072):
        nb = S // bs
        for B in (1, 4, 16):
            # enough independent caches that consecutive launches do not find their data in the 256 MB cache
            kv_bytes = B * Hkv * S * d * 2 * 2
            copies = max(1, min(8, (1 << 30) // kv_bytes))
            caches = [(synth.randn_bf16((B, Hkv, S, d), dev, gen), synth.randn_bf16((B, Hkv, S, d), dev, gen))
                      for _ in range(copies)]
            q = synth.randn_bf16((B, Hq, d), dev, gen)
            seqlens = torch.full((B,), S, dtype=torch.int32, device=dev)
            out = torch.empty(B, Hq, d, dtype=torch.bfloat16, device=dev)
            lse = torch.empty(B, Hq, dtype=torch.float32, device=dev)
            ws = torch.empty(seer.decode_workspace_bytes(B, Hq, Hkv, d, nb), dtype=torch.uint8, device=dev)

            def dense(i):
                k, v = caches[i % copies]
                seer.dense_decode(q, k, v, seqlens, nb, bs, scale, out=out, lse=lse, workspace=ws)

            t_dense = kernel_us(dense, max(4, min(args.steps, 30) // 2))
            dense_gbps = kv_bytes / (t_dense * 1e-6) / 1e9
            for sp in (0.5, 0.75, 0.9):
                k_sel = max(1, round(nb * (1 - sp)))
                lists = [synth.random_block_lists(B, Hkv, [nb] * B, [k_sel] * B, k_sel, gcpu) for _ in range(4)]
                lists = [(a.to(dev), b.to(dev)) for a, b in lists]

                def sparse(i):
                    k, v = caches[i % copies]
                    idx, cnt = lists[i % 4]
                    seer.sparse_decode(q, k, v, seqlens, idx, cnt, bs, scale, out=out, lse=lse, workspace=ws)

                time.sleep(0.2)
                t_sp = kernel_us(sparse, min(args.steps, 30))
                sel_bytes = B * Hkv * k_sel * bs * d * 2 * 2
                print(f"| {S} | {B} | {sp} | {k_sel} of {nb} | {t_dense:.1f} | {dense_gbps:.0f} | {t_sp:.1f} | "
                      f"{sel_bytes / (t_sp * 1e-6) / 1e9:.0f} | {t_dense / t_sp:.2f}x | {nb / k_sel:.2f}x |", flush=True)
            del caches
            torch.cuda.empty_cache()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="c4")
    ap.add_argument("--rotate", type=int, default=4, help="independent query sets cycled through the steps")
    ap.add_argument("--kv-copies", type=int, default=0, help="independent KV caches cycled (0 = auto)")
    ap.add_argument("--impl", type=int, default=0, help="0 auto, 1 VALU kernel, 2 MFMA kernel")
    ap.add_argument("--splits", type=int, default=0)
    ap.add_argument("--gate-impl", type=int, default=0, help="0 auto, 1 two kernels, 2 fused")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample", type=int, default=128, help="groups the CPU oracle is timed on")
    ap.add_argument("--calibrate-copy-mib", type=int, default=0,
                    help="also run a plain device copy of this many MiB (reference for hardware counters)")
    ap.add_argument("--dense-steps", type=int, default=5, help="timed dense flash-decode steps (0 = skip the dense baseline)")
    ap.add_argument("--train-tokens", type=int, default=16384,
                    help="sequence length of the training-side forward (ground-truth kernel) leg, 0 = skip")
    ap.add_argument("--also", default="c2,c3,c1,c5",
                    help="further workloads reported compactly in the same line, comma-separated ('' = none); "
                         "c1 = latency entry, c5 = the selection-mode / sparsity sweep")
    ap.add_argument("--sweep-steps", type=int, default=40, help="timed steps per point of the c5 sweep")
    ap.add_argument("--sweep-blocks", default="64,128")
    ap.add_argument("--sweep-keep", default="0.5,0.25,0.1,0.05")
    ap.add_argument("--print-sources-hash", action="store_true", help="print the kernel-source fingerprint and exit")
    ap.add_argument("--paper-sweep", action="store_true",
                    help="instead of the JSON line, print the kernel speed-up table in the shape of the paper's "
                         "kernel evaluation (8k-128k tokens, batch 1-16, sparsity 0.5-0.9; --steps launches per point)")
    args = ap.parse_args()
    if args.print_sources_hash:
        print(kernel_sources_hash())
        return
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (every box has one); --gpus must be 1. "
                 "The path shards over (batch, kv-head) groups without any communication.")

    import numpy as np
    import torch

    import paper_2506_08889_amd as seer
    import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    seer.load_library()
    if args.paper_sweep:
        paper_sweep(args, seer, synth, torch)
        return
    result = main_workload(args, seer, synth, torch, np)
    also = {}
    for name in [n for n in args.also.split(",") if n and n != args.workload]:
        time.sleep(2)      # the dense passes of the previous workload leave the GPU hot; let the clocks settle
        torch.cuda.empty_cache()
        if name == "c1":
            also["c1"] = c1_latency(args, seer, synth, torch)
        elif name == "c5":
            also["c5_sweep"] = c5_sweep(args, seer, synth, torch, [int(x) for x in args.sweep_blocks.split(",") if x],
                                        [float(x) for x in args.sweep_keep.split(",") if x])
        else:
            also[name] = also_workload(args, name, seer, synth, torch)
    if also:
        result["also"] = also
    print(json.dumps(result), flush=True)
    parity = result.get("parity_on_sample")
    if parity is not None and not parity["ok"]:
        sys.exit("bench.py: the GPU result of the sampled groups does not match the CPU oracle: " + json.dumps(parity))


if __name__ == "__main__":
    main()
