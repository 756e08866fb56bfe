#!/usr/bin/env python3
"""Benchmark of the Chorus hot path on one MI355X.

One "step" = one whole request of the 4-step Chorus schedule on the Wan2.1-1.3B-
shaped 480p model (30 blocks): projection of the prompt embedding to the model width,
the timestep modulation rows of the four noise levels, cache lookup over 4096 x 4096-d
embeddings, schedule, stage-1 full reuse of the matched latent, one stage-2 step on a
contiguous 40% box of the tokens with TGAA amplification 1.5, blend with the cached
latent, two stage-3 full steps. Inputs are synthetic, seeded, and resident in HBM
before the clock starts.

Prints ONE JSON line. `value` is milliseconds per request. `roofline` is for the
dominant kernel (self-attention): algorithmic FLOPs (4 Ls^2 D per launch) over the
launch durations measured with HIP events inside the timed region. `cpu_baseline` is
the numpy oracle timed on the host on a bounded sample, scaled to the same unit.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16
HBM_PEAK_GBS = 8000.0
# Bytes that leave / enter L2 per self-attention launch of the default workload (stage-2
# launches at 13104 tokens and stage-3 launches at 32760 tokens, weighted 30:60). Hardware
# counters cannot be read inside this process: the figure is the one the two rocprofv3 --pmc
# runs (FETCH_SIZE, then WRITE_SIZE) of this same command gave when the summary named below
# was written (FETCH_SIZE scaled by 1.992, the factor a plain 8.39 MB copy kernel of the same
# run shows; WRITE_SIZE by 1.000); it is reported for that exact workload only, with its source.
SELF_ATTN_TRAFFIC_BYTES_DEFAULT = 7.75e8
SELF_ATTN_TRAFFIC_SOURCE = "profiles/bench_wan1p3b_480p_pmc_traffic.txt"


def block_flops(Ls, D, F, Lt):
    """Algorithmic FLOPs of one block on Ls tokens (exp not counted)."""
    return 4.0 * Ls * Ls * D + 2.0 * Ls * D * (6 * D + 2 * F) + 4.0 * Ls * Lt * D + 4.0 * Lt * D * D


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="wan1p3b_480p", choices=["wan1p3b_480p", "wan1p3b_small", "c1", "wan14b_720p"])
    ap.add_argument("--blocks", type=int, default=None, help="override the block count (default: the model's)")
    ap.add_argument("--cache-entries", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--region", type=float, default=0.4, help="stage-2 region fraction (box mask)")
    ap.add_argument("--bernoulli", action="store_true", help="i.i.d. per-token mask instead of a box")
    ap.add_argument("--plain", action="store_true", help="also time a request with no reuse (4 full steps)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no collectives are part of it); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import synth
    import paper_2604_04451_amd as P
    from paper_2604_04451_amd import binding as B

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    P.load()
    dev = "cuda"
    torch.cuda.set_device(0)
    bs = synth.SHAPES[args.workload]
    n_blocks = bs.blocks if args.blocks is None else args.blocks
    N = bs.cache_N if args.cache_entries is None else args.cache_entries
    D, F, Lt, L = bs.D, bs.F, bs.Lt, bs.L
    n_steps = 4
    gen = torch.Generator(device=dev)
    gen.manual_seed(0)

    def randn(shape, std, dtype=torch.float32):
        t = torch.empty(shape, dtype=torch.float32, device=dev)
        t.normal_(0.0, std, generator=gen)
        return t.to(dtype)

    # ---- weights (random init ~N(0, 0.02), stored bf16), generated on the device
    blocks = []
    for _ in range(n_blocks):
        t = {
            "mod_table": randn((6, D), 0.02),
            "w_qkv": randn((3 * D, D), 0.02, torch.bfloat16), "b_qkv": torch.zeros(3 * D, device=dev),
            "g_q": torch.ones(D, device=dev), "g_k": torch.ones(D, device=dev),
            "w_o": randn((D, D), 0.02, torch.bfloat16), "b_o": torch.zeros(D, device=dev),
            "ln3_w": torch.ones(D, device=dev), "ln3_b": torch.zeros(D, device=dev),
            "w_cq": randn((D, D), 0.02, torch.bfloat16), "b_cq": torch.zeros(D, device=dev),
            "w_ckv": randn((2 * D, D), 0.02, torch.bfloat16), "b_ckv": torch.zeros(2 * D, device=dev),
            "g_cq": torch.ones(D, device=dev), "g_ck": torch.ones(D, device=dev),
            "w_co": randn((D, D), 0.02, torch.bfloat16), "b_co": torch.zeros(D, device=dev),
            "w_1": randn((F, D), 0.02, torch.bfloat16), "b_1": torch.zeros(F, device=dev),
            "w_2": randn((D, F), 0.02, torch.bfloat16), "b_2": torch.zeros(D, device=dev),
        }
        blocks.append(B.DeviceBlock(t, B.BlockWeights(**{n: t[n].data_ptr() for n in B._W_FIELDS})))
    arr = B.block_array(blocks)
    Pd = bs.patch_dim
    gt = {
        "w_patch": randn((D, Pd), 0.02, torch.bfloat16), "b_patch": torch.zeros(D, device=dev),
        "w_head": randn((Pd, D), 0.02, torch.bfloat16), "b_head": torch.zeros(Pd, device=dev),
        "head_table": randn((2, D), 0.02),
        "w_text1": randn((D, bs.text_dim), 0.02, torch.bfloat16), "b_text1": torch.zeros(D, device=dev),
        "w_text2": randn((D, D), 0.02, torch.bfloat16), "b_text2": torch.zeros(D, device=dev),
    }
    glue = B.DeviceGlue(gt, B.GlueWeights(**{n: gt[n].data_ptr() for n in ("w_patch", "b_patch", "w_head", "b_head", "head_table")}))
    shape = P.make_block_shape(D, bs.H, bs.dh, F, Lt, bs.grid)
    model = B.make_model_shape(shape, bs.latent_shape, (2, 2), n_blocks)

    # ---- request inputs
    text_raw = randn((Lt, bs.text_dim), bs.text_std, torch.bfloat16)
    freq_dim = 256
    tt = {
        "w_t1": randn((D, freq_dim), 0.02, torch.bfloat16), "b_t1": randn((D,), 0.02),
        "w_t2": randn((D, D), 0.02, torch.bfloat16), "b_t2": randn((D,), 0.02),
        "w_tp": randn((6 * D, D), 0.02, torch.bfloat16), "b_tp": randn((6 * D,), 0.02),
    }
    tw = B.DeviceTime.__new__(B.DeviceTime)
    tw.tensors, tw.freq_dim, tw.D = tt, freq_dim, D
    tw.cstruct = B.TimeWeights(*[tt[n].data_ptr() for n in ("w_t1", "b_t1", "w_t2", "b_t2", "w_tp", "b_tp")])
    ctx = torch.empty(Lt, D, dtype=torch.bfloat16, device=dev)
    t_mods = torch.empty(n_steps, 6, D, device=dev)
    t_heads = torch.empty(n_steps, 2, D, device=dev)
    sigmas = [1.0 - i / n_steps for i in range(n_steps + 1)]
    timesteps = [1000.0 * sg for sg in sigmas[:n_steps]]       # the model's timestep value at each noise level
    noise = randn(bs.latent_shape, 1.0)
    cache_np = synth.cache_embeddings(N, bs.cache_d, seed=0)
    near = (N * 5) // 8
    query = torch.from_numpy(synth.cache_query(cache_np, seed=0, near=near)).to(dev)
    cache_emb = torch.from_numpy(cache_np).to(dev)
    cache_lat = torch.empty((N,) + bs.latent_shape, dtype=torch.float32, device=dev)
    for i0 in range(0, N, 256):                             # 34 GB at the full shape: fill in slabs
        cache_lat[i0:i0 + 256].normal_(0.0, 1.0, generator=gen)
    T, Hg, Wg = bs.grid
    if args.bernoulli:
        mask_np = synth.bernoulli_mask(L, args.region, seed=0)
    else:
        # contiguous spatial box over all frames covering ~region of the tokens (exactly 40% by default)
        boxes = {0.1: (12, 13), 0.25: (15, 26), 0.4: (24, 26), 0.5: (30, 26), 0.75: (30, 39), 0.9: (27, 52)}
        if (Hg, Wg) == (30, 52) and args.region in boxes:
            bh, bw = boxes[args.region]
        elif (Hg, Wg) == (45, 80) and args.region == 0.5:
            bh, bw = 45, 40                                 # the 720p workload's 50 % box
        else:
            bh = max(1, int(round(Hg * args.region ** 0.5)))
            bw = max(1, int(round(Wg * args.region * Hg / bh))) if bh else 1
            bw = min(bw, Wg)
        mask_np = synth.box_mask(bs.grid, T, bh, bw, 0, (Hg - bh) // 2, (Wg - bw) // 2)
    mask = torch.from_numpy(mask_np).to(dev)
    Ls = int(mask_np.sum())
    tdiff = torch.ones(Lt, dtype=torch.uint8, device=dev)   # amplification on all text tokens
    sched = dict(gamma_override=1.5)
    latent = torch.empty_like(noise)
    lib = P.load()
    ws = torch.empty(B.chorus_denoise_run_workspace_bytes(model, N), dtype=torch.uint8, device=dev)
    ws_text = torch.empty(max(lib.chorus_text_project_workspace_bytes(Lt, D), 256), dtype=torch.uint8, device=dev)
    ws_time = torch.empty(max(lib.chorus_time_mod_workspace_bytes(D, freq_dim), 256), dtype=torch.uint8, device=dev)

    def request(tau=0.75):
        """Everything a request computes, from the raw prompt embedding and the initial noise to the final latent."""
        B.chorus_stage1_copy(latent, noise)
        B.chorus_text_project(text_raw, glue, ctx, ws_text)
        for i in range(n_steps):
            B.chorus_time_mod(timesteps[i], tw, t_mods[i], t_heads[i], ws_time)
        return B.chorus_denoise_run(model, arr, glue, latent, cache_emb, cache_lat.unsqueeze(1), query, tau, sigmas, t_mods, t_heads,
                                    ctx, tdiff=tdiff, mask_see=mask, mask_edit=mask, sched=sched, ws=ws,
                                    latent_steps=[1])       # every entry holds the latent after one step

    # warm-up; the first pass runs with the profiler on so that its event pool exists before the clock starts
    B.prof_reset()
    B.prof_enable([B.PROF_SELF_ATTN])
    for _ in range(max(args.warmup, 1)):
        res = request()
    torch.cuda.synchronize()
    B.prof_reset()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        res = request()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    attn_ms, attn_n = B.prof_read(B.PROF_SELF_ATTN)
    B.prof_enable([])
    B.prof_reset()
    ms = (t1 - t0) * 1e3 / max(args.steps, 1)
    assert res["hit"] and res["index"] == near and (res["K1"], res["K2"]) == (1, 2) and res["Ls"] == Ls, res
    # the result of the last timed request: finite everywhere, the cached latent bit for bit outside the region
    # (Eq. 6 ... then two full steps move every token), and different from the initial noise
    assert bool(torch.isfinite(latent).all()), "non-finite latent"
    assert float((latent - noise).abs().max()) > 1e-3 and float((latent - cache_lat[near]).abs().max()) > 1e-3

    # ---- roofline of the dominant kernel: self-attention, 4 Ls^2 D FLOPs per launch
    default_workload = (args.workload == "wan1p3b_480p" and args.blocks is None and args.cache_entries is None
                        and args.region == 0.4 and not args.bernoulli)
    per_req_attn_flops = n_blocks * (4.0 * Ls * Ls * D + 2 * 4.0 * L * L * D)
    attn_tflops = per_req_attn_flops * args.steps / (attn_ms * 1e-3) / 1e12 if attn_ms > 0 else 0.0
    plan_flops = n_blocks * (block_flops(Ls, D, F, Lt) + 2 * block_flops(L, D, F, Lt))
    out = {
        # the metric's name is the one the baseline file gives for the default workload; another workload says so
        "metric": ("ms per 4-step video denoise + self-attn TFLOP/s, Wan-1.3B-shape 480p block" if args.workload == "wan1p3b_480p"
                   else f"ms per 4-step video denoise + self-attn TFLOP/s, workload {args.workload}"),
        "value": round(ms, 3), "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 3), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{bs.name}: 4-step Chorus schedule, {n_blocks} blocks, L={L}, D={D}, H={bs.H}x{bs.dh}, "
                               f"F={F}, Lt={Lt}, cache {N}x{bs.cache_d}, stage-2 "
                               f"{'bernoulli' if args.bernoulli else 'box'} mask {Ls}/{L} tokens, TGAA 1.5; "
                               f"text projection and timestep modulation inside the request",
                   "stages": [1, 2, 3, 3], "blocks": n_blocks, "tokens": L, "stage2_tokens": Ls},
        "request_tflops": round(plan_flops / (ms * 1e-3) / 1e12, 2),
        "self_attn_tflops": round(attn_tflops, 2),
        "self_attn_ms_per_launch": round(attn_ms / max(attn_n, 1), 4),
        "roofline": {"bound": "mfma", "achieved": round(attn_tflops, 2), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(attn_tflops / MFMA_BF16_PEAK_TFLOPS, 4),
                     "traffic": (SELF_ATTN_TRAFFIC_BYTES_DEFAULT if default_workload else None),
                     "traffic_source": (SELF_ATTN_TRAFFIC_SOURCE if default_workload else None),
                     # Q, K, V read once and O written once per launch, averaged over the request's launches
                     # (one per block at the stage-2 token count, two per block at the full count)
                     "algorithmic_bytes": (4 * 2.0 * Ls * D + 2 * 4 * 2.0 * L * D) / 3.0,
                     "kernel": "attention_pp16_kernel<128,true,2,0> (self-attention; at 13104 tokens its last, partly filled round runs as attention_pp16_kernel<128,true,1,0>)", "launches": attn_n},
    }
    # what a bare MFMA loop sustains on this device right now (the part is power-managed: the rate depends on the
    # operand values and on the LDS reads and exponentials that accompany the MFMAs); context for roofline.frac
    out["mfma_ceiling_tflops"] = {
        "ones_registers_only": round(B.chorus_mfma_ceiling(False, 0, 20), 1),
        "normal_registers_only": round(B.chorus_mfma_ceiling(True, 0, 20), 1),
        "normal_lds_operand": round(B.chorus_mfma_ceiling(True, 1, 20), 1),
        "normal_lds_operand_exp2": round(B.chorus_mfma_ceiling(True, 3, 20), 1),
    }
    # and what a plain streaming copy sustains (read + write of 2 x 268 MB, rotating buffers), for the HBM-bound steps
    cp = [torch.empty(2, 67108864, dtype=torch.float32, device=dev) for _ in range(3)]
    for i in range(6):
        B.chorus_stage1_copy(cp[i % 3][1], cp[i % 3][0])
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(30):
        B.chorus_stage1_copy(cp[i % 3][1], cp[i % 3][0])
    e1.record()
    torch.cuda.synchronize()
    out["hbm_copy_ceiling_gbs"] = round(30 * 2 * 67108864 * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
    del cp
    if args.plain:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        request(tau=2.0)   # no cache entry can reach this threshold: 4 full steps
        torch.cuda.synchronize()
        out["plain_4_step_ms"] = round((time.perf_counter() - t0) * 1e3, 3)

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(bs, n_blocks, L, Ls)
    print(json.dumps(out), flush=True)


def cpu_baseline(bs, n_blocks, L, Ls):
    """The numpy fp64 oracle, as it stands, timed on one block of the same widths at the two largest of the token
    counts 2048, 4096, 8192 that fit in about 20 s of host time (TGAA 1.5 as in the stage-2 step). A block costs
    a L + b L^2 (per-token work and self-attention); the two timings fix a and b, and the request is
    n_blocks * (cost(Ls) + 2 cost(L)): an extrapolation, labelled as such."""
    import dataclasses
    import synth
    from oracle import chorus_oracle as O
    w = synth.block_weights(bs, 0)
    times = []
    # grow the sample while the host keeps up: 2048 tokens, then 4096, then 8192 if the first two took under 8 s
    for grid in ([bs.grid] if bs.L <= 4096 else [(2, 32, 32), (4, 32, 32), (8, 32, 32)]):
        if len(times) == 2 and sum(t for _, t in times) > 8.0:
            break
        small = dataclasses.replace(bs, grid=grid)
        inp = synth.block_inputs(small, 0)
        t0 = time.perf_counter()
        O.dit_block(inp["x"], w, small, inp["text_ctx"], inp["t_mod"], key_scale=np.full(small.Lt, 1.5), gamma_o=1.5)
        times.append((small.L, time.perf_counter() - t0))
    times = times[-2:]
    if len(times) == 2:
        (l1, t1), (l2, t2) = times
        b = (t2 / l2 - t1 / l1) / (l2 - l1)
        a = t1 / l1 - b * l1
        b = max(b, 0.0)
    else:
        (l1, t1), = times
        a, b = t1 / l1, 0.0
    cost = lambda n: a * n + b * n * n
    total = n_blocks * (cost(Ls) + 2 * cost(L))
    try:
        import threadpoolctl
        info = threadpoolctl.threadpool_info()
        cores = max(p["num_threads"] for p in info) if info else 1
    except Exception:
        cores = os.cpu_count() or 1
    fl = block_flops(times[-1][0], bs.D, bs.F, bs.Lt)
    return {"value": round(total * 1e3, 1), "unit": "ms per 4-step denoise (extrapolated from two measured block sizes)",
            "cores": int(cores), "kind": "oracle",
            "sample": "one block of the same widths, measured at " + " and ".join(f"{l} tokens: {t:.2f} s" for l, t in times)
                      + f" ({fl / times[-1][1] / 1e9:.0f} GFLOP/s fp64 at the larger; self-attention is "
                      + f"{4.0 * times[-1][0] ** 2 * bs.D / fl:.0%} of its FLOPs, {b * times[-1][0] ** 2 / max(times[-1][1], 1e-9):.0%} of its time); "
                      + f"block cost a*L + b*L^2 fitted to the two, request = {n_blocks} x (cost({Ls}) + 2 cost({L}))"}


if __name__ == "__main__":
    main()
