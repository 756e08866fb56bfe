"""Helpers shared by the GPU parity tests: host<->device conversion and error metrics."""
import numpy as np
import torch

import synth

DEV = "cuda"

# spec tolerances for floating point (bf16 GPU path against the fp64 oracle)
MAX_ABS = 2e-2
REL_L2 = 5e-3


def dev_f32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV)


def dev_bf16(a):
    """numpy fp32 (bf16-representable or not) -> device bf16 via one RNE rounding done in numpy."""
    bits = synth.to_bf16_bits(np.ascontiguousarray(a, dtype=np.float32)).reshape(np.shape(a))
    return torch.from_numpy(bits.view(np.int16)).to(DEV).view(torch.bfloat16)


def host_bf16(t):
    """device bf16 tensor -> numpy float64"""
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def host(t):
    return t.detach().cpu().numpy()


def errs(got, ref):
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    max_abs = float(np.abs(got - ref).max()) if got.size else 0.0
    den = float(np.linalg.norm(ref))
    rel = float(np.linalg.norm(got - ref) / den) if den > 0 else float(np.linalg.norm(got - ref))
    return max_abs, rel


def check(got, ref, name, max_abs=MAX_ABS, rel_l2=REL_L2):
    assert np.isfinite(np.asarray(got, np.float64)).all(), f"{name}: non-finite output"
    a, r = errs(got, ref)
    print(f"[parity] {name}: max_abs={a:.3e} rel_l2={r:.3e}", flush=True)
    assert a <= max_abs, f"{name}: max-abs {a:.3e} > {max_abs}"
    assert r <= rel_l2, f"{name}: rel-L2 {r:.3e} > {rel_l2}"
    return a, r
