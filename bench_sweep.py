#!/usr/bin/env python3
"""Kernel speed-up sweep in the shape of the paper's kernel evaluation (Sec. 4.4): random tensors,
64 query / 8 kv heads, head dim 128, block 64; sequence length 8k..128k, batch 1..16, block sparsity
0.5 / 0.75 / 0.9 (uniformly random block lists, the same count for every group).  For every point
the block-sparse decode (split kernel + merge) and the dense flash-decode of this library are timed
with HIP events through the library's own per-kernel timers; prints a markdown table.

    python bench_sweep.py [--iters 20] > table.md
"""
from __future__ import annotations

import argparse
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--iters", type=int, default=20)
    ap.add_argument("--heads", type=int, default=64)
    ap.add_argument("--kv-heads", type=int, default=8)
    args = ap.parse_args()
    import torch

    import paper_2506_08889_amd as seer
    import synth

    dev = "cuda:0"
    Hq, Hkv, d, bs = args.heads, args.kv_heads, 128, 64
    scale = 1.0 / d ** 0.5
    gen = synth.generator(dev, 7)
    gcpu = torch.Generator().manual_seed(7)

    def kernel_us(fn, n):
        for i in range(3):
            fn(i)
        seer.profile_reset()
        seer.profile_enable(True)
        for i in range(n):
            fn(i)
        torch.cuda.synchronize()
        seer.profile_enable(False)
        ns, ts = seer.profile_read(2)
        nm, tm = seer.profile_read(3)
        seer.profile_reset()
        return (ts / ns + (tm / nm if nm else 0.0)) * 1e3

    print(f"| seqlen | batch | sparsity | selected blocks | dense us | dense GB/s | sparse us | sparse GB/s | speed-up | ideal |")
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

            t_dense = kernel_us(dense, max(4, args.iters // 2))
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
                t_sp = kernel_us(sparse, args.iters)
                sel_bytes = B * Hkv * k_sel * bs * d * 2 * 2
                print(f"| {S} | {B} | {sp} | {k_sel} of {nb} | {t_dense:.1f} | {dense_gbps:.0f} | {t_sp:.1f} | "
                      f"{sel_bytes / (t_sp * 1e-6) / 1e9:.0f} | {t_dense / t_sp:.2f}x | {nb / k_sel:.2f}x |", flush=True)
            del caches
            torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
