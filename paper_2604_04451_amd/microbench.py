"""Per-entry-point timing of the memory-bound steps of the Chorus hot path on one MI355X:
cache lookup, stage-1 copy, latent fusion, compaction, row gather / scatter, the
region-mask pipeline and the per-token normalisation kernels, at the Wan2.1-1.3B 480p
shapes; then the matrix-pipe ceiling this device sustains (a bare MFMA loop, by operand
data and by what accompanies the MFMAs). Each call is timed with HIP events on the launch stream over a rotation of
buffers larger than the last-level cache, so every launch reads cold data.

    python -m paper_2604_04451_amd.microbench [--iters 48]

Prints one line per entry point: algorithmic bytes, median and best microseconds, and
the rate on algorithmic bytes. Run it under `rocprofv3 --kernel-trace --stats` for the
per-kernel durations without launch overhead.
"""
from __future__ import annotations

import argparse

import numpy as np
import torch

from . import binding as B

DEV = "cuda"


def timeit(fn, n):
    for i in range(3):
        fn(i)
    torch.cuda.synchronize()
    ts = []
    for i in range(n):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn(i)
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1) * 1e3)
    return float(np.median(ts)), float(min(ts))


def report(name, nbytes, med, best):
    print(f"{name:<44s} {nbytes / 1e6:9.3f} MB  median {med:7.1f} us  best {best:7.1f} us  "
          f"{nbytes / med / 1e3:7.0f} GB/s median  {nbytes / best / 1e3:7.0f} GB/s best", flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--iters", type=int, default=48)
    args = ap.parse_args()
    n = args.iters
    if not torch.cuda.is_available():
        raise SystemExit("microbench: needs a GPU")
    B.load()
    g = torch.Generator(device=DEV)
    g.manual_seed(0)

    # ---- lookup: 10 caches of 67 MB, more than the 256 MB last-level cache
    N = d = 4096
    caches = [torch.randn(N, d, device=DEV, generator=g) for _ in range(10)]
    q = torch.randn(d, device=DEV, generator=g)
    out = torch.empty(3, dtype=torch.int32, device=DEV)
    ws = torch.empty(1 << 16, dtype=torch.uint8, device=DEV)
    med, best = timeit(lambda i: B.chorus_cache_lookup(caches[i % 10], q, 0.75, out, ws), n)
    report("cache_lookup 4096x4096 fp32 (2 launches)", N * d * 4 + d * 4, med, best)
    # the same scan for a batch of queries with top-8 candidates each (the cache is streamed once per 32 queries)
    for Q in (1, 16, 32):
        qs = torch.randn(Q, d, device=DEV, generator=g)
        wsb = torch.empty(B.load().chorus_cache_lookup_batch_workspace_bytes(N, d, Q), dtype=torch.uint8, device=DEV)
        med, best = timeit(lambda i: B.chorus_cache_lookup_batch(caches[i % 10], qs, 0.75, 8, wsb), n)
        report(f"cache_lookup_batch Q={Q} k=8 (2 launches)", N * d * 4 + Q * d * 4, med, best)
    # the scan over a low-precision copy with the exact re-rank (3 launches): a query near an entry (one row is
    # re-scored) and one far from every entry (bf16: a handful; FP8: its proven margin keeps every row, the re-rank
    # then is a whole fp32 scan)
    for fmt, name, eb in ((B.LP_BF16, "bf16", 2), (B.LP_FP8, "fp8", 1)):
        lps = [B.chorus_cache_lowprec_store(c, fmt) for c in caches]
        wsl = torch.empty(B.load().chorus_cache_lookup_lowprec_workspace_bytes(N), dtype=torch.uint8, device=DEV)
        nres = torch.empty(1, dtype=torch.int32, device=DEV)
        for qname, qq in (("near an entry", [c[123] + 0.3 * torch.randn(d, device=DEV, generator=g) for c in caches]),
                          ("far from all", [torch.randn(d, device=DEV, generator=g) for _ in caches])):
            med, best = timeit(lambda i: B.chorus_cache_lookup_lowprec(caches[i % 10], lps[i % 10], fmt, qq[i % 10], 0.75, out, nres, wsl), n)
            k = int(nres.cpu()[0])
            report(f"cache_lookup_lowprec {name}, query {qname} ({k} re-scored)", N * d * eb + k * d * 4 + d * 4, med, best)
        del lps
    del caches

    # ---- latent-sized kernels: 24 triples of 8.4 MB
    C_, T, Hl, Wl = 16, 21, 60, 104
    Hg, Wg = Hl // 2, Wl // 2
    L = T * Hg * Wg
    bufs = [torch.randn(3, C_, T, Hl, Wl, device=DEV, generator=g) for _ in range(24)]
    lat_bytes = bufs[0][0].numel() * 4
    box = torch.zeros(T, Hg, Wg, dtype=torch.uint8, device=DEV)
    box[:, 3:27, 13:39] = 1                                                 # 21 x 24 x 26 = 40 %
    bern = (torch.rand(L, device=DEV, generator=g) < 0.5).to(torch.uint8)
    for name, m in (("box 40 %", box.reshape(-1)), ("Bernoulli 50 %", bern)):
        med, best = timeit(lambda i: B.chorus_region_blend(bufs[i % 24][2], bufs[i % 24][0], bufs[i % 24][1], m), n)
        report(f"region_blend {name}", 2 * lat_bytes + L, med, best)
    med, best = timeit(lambda i: B.chorus_stage1_copy(bufs[i % 24][2], bufs[i % 24][0]), n)
    report("stage1_copy", 2 * lat_bytes, med, best)
    # the same kernels on 16 latents per call (C = 256 planes): large enough to leave the launch floor behind
    big = [torch.randn(3, 16 * C_, T, Hl, Wl, device=DEV, generator=g) for _ in range(3)]
    for name, m in (("box 40 %", box.reshape(-1)), ("Bernoulli 50 %", bern)):
        med, best = timeit(lambda i: B.chorus_region_blend(big[i % 3][2], big[i % 3][0], big[i % 3][1], m), n)
        report(f"region_blend {name}, 16 latents per call", 16 * (2 * lat_bytes) + L, med, best)
    med, best = timeit(lambda i: B.chorus_stage1_copy(big[i % 3][2], big[i % 3][0]), n)
    report("stage1_copy, 16 latents per call", 32 * lat_bytes, med, best)
    del big

    # ---- compaction and row moves
    idx = torch.empty(L, dtype=torch.int32, device=DEV)
    cnt = torch.empty(1, dtype=torch.int32, device=DEV)
    med, best = timeit(lambda i: B.chorus_region_compact(box.reshape(-1), idx, cnt, ws), n)
    Ls = int(cnt.cpu()[0])
    report("region_compact box 40 % (3 launches)", L + 4 * Ls, med, best)
    W = 64
    rows = [torch.randn(2, L, W, device=DEV, generator=g) for _ in range(24)]
    med, best = timeit(lambda i: B.chorus_region_gather_rows(rows[i % 24][1], rows[i % 24][0], idx, Ls), n)
    report("region_gather_rows W=64 fp32, 40 %", 2 * Ls * W * 4 + 4 * Ls, med, best)
    med, best = timeit(lambda i: B.chorus_region_scatter_rows(rows[i % 24][1], rows[i % 24][0], idx, Ls), n)
    report("region_scatter_rows W=64 fp32, 40 %", 2 * Ls * W * 4 + 4 * Ls, med, best)
    del rows, bufs

    # ---- region masks: 21 key frames of 480 x 832, 81 frames, window 4 x 16 x 16 -> 21 x 30 x 52
    Tp, Kf, Hp, Wp = 81, 21, 480, 832
    kms = [(torch.rand(Kf, Hp, Wp, device=DEV, generator=g) < 0.001).to(torch.uint8) for _ in range(40)]
    fk = torch.minimum(torch.arange(Tp, device=DEV) * Kf // Tp, torch.tensor(Kf - 1, device=DEV)).to(torch.int32)
    base = torch.empty(T, Hg, Wg, dtype=torch.uint8, device=DEV)
    med, best = timeit(lambda i: B.chorus_mask_project(kms[i % 40], fk, Tp, (4, 16, 16), 1, base), n)
    report("mask_project 21x480x832 -> 21x30x52", Kf * Hp * Wp + L + 4 * Tp, med, best)
    del kms
    med, best = timeit(lambda i: B.chorus_mask_hierarchy(box, (0, 1, 1), (1, 3, 3)), n)
    report("mask_hierarchy 21x30x52 r=(0,1,1) r'=(1,3,3)", 3 * L, med, best)

    # ---- per-token normalisation kernels at L = 32760, D = 1536 (rotation of 4: 0.2-0.6 GB each)
    D, H, dh = 1536, 12, 128
    Lpad = (L + 255) // 256 * 256
    xs = [torch.randn(L, D, device=DEV, generator=g) for _ in range(4)]
    hs = [torch.empty(L, D, dtype=torch.bfloat16, device=DEV) for _ in range(4)]
    vec = [torch.randn(D, device=DEV, generator=g) * 0.02 for _ in range(4)]
    med, best = timeit(lambda i: B.chorus_ln_modulate(xs[i % 4], hs[i % 4], vec[0], vec[1], vec[2], vec[3], True), n)
    report("ln_modulate 32760x1536", L * D * 6, med, best)
    qkv = [torch.randn(L, 3 * D, device=DEV, generator=g).to(torch.bfloat16) for _ in range(4)]
    qo = [torch.empty(H, Lpad, dh, dtype=torch.bfloat16, device=DEV) for _ in range(4)]
    vt = [torch.empty(D, Lpad, dtype=torch.bfloat16, device=DEV) for _ in range(4)]
    tok = torch.arange(L, dtype=torch.int32, device=DEV)
    gain = torch.ones(D, device=DEV)
    med, best = timeit(lambda i: B.chorus_qk_norm_rope(qkv[i % 4], 0, gain, qo[i % 4], L, H, dh, tok, (T, Hg, Wg), True), n)
    report("qk_norm_rope 32760x1536 (one of q, k)", L * D * 4, med, best)
    med, best = timeit(lambda i: B.chorus_v_transpose(qkv[i % 4], 2 * D, vt[i % 4], L), n)
    report("v_transpose 32760x1536", L * D * 4, med, best)

    # ---- self-attention at the 480p length on N(0,1) operands and on constant ones: same launches, same instruction
    #      stream, different power draw
    Q = torch.empty(H, Lpad, dh, dtype=torch.bfloat16, device=DEV)
    K = torch.empty(H, Lpad, dh, dtype=torch.bfloat16, device=DEV)
    Vt = torch.empty(D, Lpad, dtype=torch.bfloat16, device=DEV)
    Oo = torch.empty(L, D, dtype=torch.bfloat16, device=DEV)
    # the kernel the block launches at this length: variant 6, queries pre-multiplied by log2(e) / sqrt(dh)
    qc = float(np.log2(np.e) / np.sqrt(dh))
    for dname in ("N(0,1)", "all 1.0"):
        for t in (Q, K, Vt):
            if dname == "all 1.0":
                t.fill_(1.0)
            else:
                t.copy_(torch.randn(t.shape, device=DEV, generator=g))
        Q.copy_(Q.float() * qc)
        for _ in range(20):
            B.chorus_attention(Q, K, Vt, Oo, None, L, L, 6)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(20):
            B.chorus_attention(Q, K, Vt, Oo, None, L, L, 6)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 20
        tf = 4.0 * L * L * D / ms / 1e9
        print(f"self_attention L={L} H={H}x{dh}, operands {dname:<8s} {ms:7.3f} ms  {tf:8.1f} TFLOP/s  "
              f"({tf / 2500.0:.3f} of 2.5 PFLOP/s)", flush=True)
    del Q, K, Vt, Oo

    # ---- what the matrix pipe sustains on this device (power-managed: depends on data and instruction mix)
    for data, dname in ((False, "operands all 1.0"), (True, "operands N(0,1)")):
        for mix, mname in ((0, "registers only"), (1, "A operand from LDS"), (2, "+ exp2 and max per logit"),
                           (3, "A from LDS + exp2")):
            tf = B.chorus_mfma_ceiling(data, mix, 20)
            print(f"mfma_ceiling bf16 16x16x32, {dname}, {mname:<28s} {tf:8.1f} TFLOP/s  ({tf / 2500.0:.3f} of 2.5 PFLOP/s)",
                  flush=True)


if __name__ == "__main__":
    main()
