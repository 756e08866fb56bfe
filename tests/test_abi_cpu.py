"""CPU-side checks of the C-ABI library: it loads, exports every function the
headers declare, validates arguments before touching the GPU, and its host-only
schedule agrees with the oracle. No kernel is launched here."""
import ctypes as C
import math
import os
import re

import numpy as np
import pytest

from oracle import chorus_oracle as O
import paper_2604_04451_amd as P
from paper_2604_04451_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    names = set()
    for h in ("chorus.h", "chorus_ops.h"):
        src = open(os.path.join(ROOT, "include", h)).read()
        src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
        names |= set(re.findall(r"\b(chorus_[a-z0-9_]+)\s*\(", src))
    return names


def test_library_exports_every_declared_symbol():
    lib = P.load()
    decl = _declared()
    assert {"chorus_cache_lookup", "chorus_dit_block_step", "chorus_region_blend", "chorus_denoise_schedule"} <= decl
    for name in sorted(decl):
        assert hasattr(lib, name), f"{name} declared in include/ but not exported"
    # and the binding knows a signature for each
    assert decl <= set(lib._sigs), sorted(decl - set(lib._sigs))
    assert lib.chorus_version() >= 100


@pytest.mark.parametrize("N", [1, 4, 5, 8, 50])
@pytest.mark.parametrize("tau", [0.65, 0.75])
def test_schedule_matches_oracle(N, tau):
    for params in (None, dict(gamma_override=1.5), dict(a1=0.1, b1=0.5, a2=0.2, b2=0.3, r3=2, Gamma_k=2.0, lam=0.9)):
        for m in list(np.linspace(0.0, 1.0, 101)) + [float("nan"), -math.inf, 1.5]:
            mf = float(np.float32(m))
            k1, k2, plan = P.chorus_denoise_schedule(mf, tau, N, params)
            ok1, ok2, oplan = O.denoise_schedule(mf, float(np.float32(tau)), N, params)
            assert (k1, k2) == (ok1, ok2), (m, tau, N, params)
            for (s, gk, go), (os_, ogk, ogo) in zip(plan, oplan):
                assert s == os_
                assert gk == np.float32(ogk) and go == np.float32(ogo)


def test_argument_validation_returns_codes():
    lib = P.load()
    null = C.c_void_p(0)
    out = (C.c_int32 * 3)()
    # lookup: d not a multiple of 4; missing workspace; negative N
    assert lib.chorus_cache_lookup(C.c_void_p(16), 4, 6, C.c_void_p(16), 0.5, out, C.c_void_p(16), 1024, null) == B.E_SHAPE
    assert lib.chorus_cache_lookup(C.c_void_p(16), 4, 8, C.c_void_p(16), 0.5, out, null, 0, null) == B.E_WORKSPACE
    assert lib.chorus_cache_lookup(C.c_void_p(16), -1, 8, C.c_void_p(16), 0.5, out, C.c_void_p(16), 1024, null) == B.E_ARG
    assert lib.chorus_cache_lookup(C.c_void_p(8), 4, 8, C.c_void_p(16), 0.5, out, C.c_void_p(16), 1024, null) == B.E_ARG
    # more entries than the int32 result index can name
    assert lib.chorus_cache_lookup(C.c_void_p(16), 1 << 31, 8, C.c_void_p(16), 0.5, out, C.c_void_p(16), 1 << 20, null) == B.E_SHAPE
    # the workspace-free lookup validates the same way, before any device call
    assert lib.chorus_cache_lookup_static(C.c_void_p(16), 4, 6, C.c_void_p(16), 0.5, out, null) == B.E_SHAPE
    assert lib.chorus_cache_lookup_static(C.c_void_p(16), -1, 8, C.c_void_p(16), 0.5, out, null) == B.E_ARG
    assert lib.chorus_cache_lookup_static(C.c_void_p(16), 1 << 31, 8, C.c_void_p(16), 0.5, out, null) == B.E_SHAPE
    assert lib.chorus_cache_lookup_static(C.c_void_p(16), 4, 8, C.c_void_p(16), 0.5, None, null) == B.E_ARG
    # low-precision storage: sizes, unknown format, width not a multiple of 16, missing workspace
    assert lib.chorus_cache_lowprec_bytes(10, 64, B.LP_BF16) == 1280 and lib.chorus_cache_lowprec_bytes(10, 64, B.LP_FP8) == 640
    assert lib.chorus_cache_lowprec_bytes(10, 64, 7) == 0
    assert lib.chorus_cache_lowprec_store(C.c_void_p(16), 4, 64, 7, C.c_void_p(16), null) == B.E_ARG
    assert lib.chorus_cache_lowprec_store(C.c_void_p(16), 4, 24, B.LP_FP8, C.c_void_p(16), null) == B.E_SHAPE
    assert lib.chorus_cache_lowprec_store(C.c_void_p(16), 0, 64, B.LP_FP8, null, null) == B.OK
    assert lib.chorus_cache_lookup_lowprec(C.c_void_p(16), C.c_void_p(16), B.LP_BF16, 4, 64, C.c_void_p(16), 0.5, out, null, null, 0, null) == B.E_WORKSPACE
    assert lib.chorus_cache_lookup_lowprec(C.c_void_p(16), C.c_void_p(16), 3, 4, 64, C.c_void_p(16), 0.5, out, null, C.c_void_p(16), 1 << 20, null) == B.E_ARG
    assert lib.chorus_cache_lookup_lowprec(C.c_void_p(16), C.c_void_p(16), B.LP_FP8, 4, 40, C.c_void_p(16), 0.5, out, null, C.c_void_p(16), 1 << 20, null) == B.E_SHAPE
    assert lib.chorus_cache_lookup_lowprec_workspace_bytes(4096) >= 4096 * 4
    # schedule
    assert lib.chorus_denoise_schedule(0.9, 0.75, -1, None, None, None, None) == B.E_ARG
    assert lib.chorus_denoise_schedule(0.9, 0.75, 0, None, None, None, None) == B.OK
    # blend: H not divisible by the patch
    assert lib.chorus_region_blend(C.c_void_p(16), C.c_void_p(16), C.c_void_p(16), C.c_void_p(16), 1, 1, 3, 4, 2, 2, null) == B.E_SHAPE
    assert lib.chorus_region_blend(null, null, null, null, 0, 1, 4, 4, 2, 2, null) == B.OK   # empty tensor
    # block: unsupported head dim, H*dh != D, missing workspace
    bad = B.BlockShape(256, 4, 32, 1024, 16, 4, 8, 8)
    w = B.BlockWeights()
    assert lib.chorus_dit_block_step(C.byref(bad), C.byref(w), C.c_void_p(16), 4, null, C.c_void_p(16), C.c_void_p(16), null, 1.0, C.c_void_p(16), 1 << 20, null) == B.E_SHAPE
    bad2 = B.BlockShape(256, 3, 64, 1024, 16, 4, 8, 8)
    assert lib.chorus_dit_block_workspace_bytes(C.byref(bad2), 10) == 0
    good = B.BlockShape(256, 4, 64, 1024, 16, 4, 8, 8)
    need = lib.chorus_dit_block_workspace_bytes(C.byref(good), 256)
    assert need > 0
    assert lib.chorus_dit_block_step(C.byref(good), C.byref(w), C.c_void_p(16), 256, null, C.c_void_p(16), C.c_void_p(16), null, 1.0, C.c_void_p(256), need - 1, null) == B.E_WORKSPACE
    assert lib.chorus_dit_block_step(C.byref(good), C.byref(w), C.c_void_p(16), 0, null, C.c_void_p(16), C.c_void_p(16), null, 1.0, null, 0, null) == B.OK  # Ls == 0
    # gemm: K not a multiple of 64
    assert lib.chorus_gemm_bf16(C.c_void_p(16), C.c_void_p(16), 8, 64, 100, 0, C.c_void_p(16), null, null, null, 1.0, null) == B.E_SHAPE
    # attention: head dim, pad
    assert lib.chorus_attention(C.c_void_p(16), C.c_void_p(16), C.c_void_p(16), C.c_void_p(16), null, 8, 8, 64, 64, 2, 96, 0, null) == B.E_SHAPE
    assert lib.chorus_attention(C.c_void_p(16), C.c_void_p(16), C.c_void_p(16), C.c_void_p(16), null, 8, 8, 64, 60, 2, 64, 0, null) == B.E_SHAPE
    assert lib.chorus_attention(C.c_void_p(16), C.c_void_p(16), C.c_void_p(16), C.c_void_p(16), null, 8, 0, 64, 64, 2, 64, 0, null) == B.E_SHAPE


def test_workspace_sizes_scale_with_rows():
    lib = P.load()
    sh = B.BlockShape(1536, 12, 128, 8960, 512, 21, 30, 52)
    a = lib.chorus_dit_block_workspace_bytes(C.byref(sh), 13104)
    b = lib.chorus_dit_block_workspace_bytes(C.byref(sh), 32760)
    assert 0 < a < b < 3 * (1 << 30)
    # the scan leaves 8 bytes per workgroup of four rows (at most 4096 workgroups) behind a 256-byte header
    assert lib.chorus_cache_lookup_workspace_bytes(4096) >= 256 + 1024 * 8
    assert lib.chorus_cache_lookup_workspace_bytes(1 << 24) == lib.chorus_cache_lookup_workspace_bytes(1 << 20) >= 256 + 4096 * 8
    assert lib.chorus_cache_lookup_workspace_bytes(0) >= 256
    assert lib.chorus_region_compact_workspace_bytes(75600) >= 4 * ((75600 + 4095) // 4096)


def test_mask_entry_points_validate_and_pooled_extent_matches_oracle():
    from oracle import chorus_oracle as O
    lib = P.load()
    null, p16 = C.c_void_p(0), C.c_void_p(16)
    for n, k, lead in [(81, 4, 1), (480, 16, 0), (17, 4, 0), (5, 7, 0), (1, 1, 1), (0, 3, 0), (9, 2, 9)]:
        assert lib.chorus_mask_pooled_extent(n, k, lead) == O.pooled_extent(n, k, lead)
    assert lib.chorus_mask_pooled_extent(8, 0, 0) == B.E_ARG
    assert lib.chorus_mask_pooled_extent(8, 2, 9) == B.E_ARG
    # project: window < 1, t_lead > Tp, identity frame map with Kf != Tp, null pointers; empty input is OK
    assert lib.chorus_mask_project(p16, 2, p16, 4, 8, 8, 0, 2, 2, 0, p16, null) == B.E_ARG
    assert lib.chorus_mask_project(p16, 2, p16, 4, 8, 8, 2, 2, 2, 5, p16, null) == B.E_ARG
    assert lib.chorus_mask_project(p16, 2, null, 4, 8, 8, 2, 2, 2, 0, p16, null) == B.E_ARG
    assert lib.chorus_mask_project(null, 2, p16, 4, 8, 8, 2, 2, 2, 0, p16, null) == B.E_ARG
    assert lib.chorus_mask_project(p16, 2, p16, 4, 8, 1 << 20, 2, 2, 2, 0, p16, null) == B.E_SHAPE
    assert lib.chorus_mask_project(null, 0, null, 0, 8, 8, 2, 2, 2, 0, null, null) == B.OK
    # hierarchy: r' < r, negative radius, aliasing, no output; empty grid is OK
    r = lambda *v: (C.c_int32 * 3)(*v)
    assert lib.chorus_mask_hierarchy(p16, 2, 4, 4, r(0, 2, 2), r(0, 1, 3), C.c_void_p(32), C.c_void_p(64), null) == B.E_ARG
    assert lib.chorus_mask_hierarchy(p16, 2, 4, 4, r(0, -1, 0), r(0, 1, 1), C.c_void_p(32), C.c_void_p(64), null) == B.E_ARG
    assert lib.chorus_mask_hierarchy(p16, 2, 4, 4, r(0, 1, 1), r(0, 1, 1), p16, C.c_void_p(64), null) == B.E_ARG
    assert lib.chorus_mask_hierarchy(p16, 2, 4, 4, r(0, 1, 1), r(0, 1, 1), null, null, null) == B.E_ARG
    assert lib.chorus_mask_hierarchy(p16, 2, 4, 4, None, r(0, 1, 1), C.c_void_p(32), C.c_void_p(64), null) == B.E_ARG
    assert lib.chorus_mask_hierarchy(null, 0, 4, 4, r(0, 1, 1), r(0, 1, 1), null, null, null) == B.OK


def test_cache_insert_validates():
    lib = P.load()
    null, p16 = C.c_void_p(0), C.c_void_p(16)
    assert lib.chorus_cache_insert(p16, p16, 8, 8, 16, 64, p16, p16, null) == B.E_ARG     # slot == capacity
    assert lib.chorus_cache_insert(p16, p16, 8, -1, 16, 64, p16, p16, null) == B.E_ARG
    assert lib.chorus_cache_insert(null, p16, 8, 0, 16, 64, p16, p16, null) == B.E_ARG
    assert lib.chorus_cache_insert(p16, p16, 8, 0, 0, 64, p16, p16, null) == B.E_ARG
    assert lib.chorus_cache_insert(p16, p16, 0, 0, 16, 64, p16, p16, null) == B.E_ARG


def _shifted_sigmas(n, shift):
    """Linear levels from 1 to 0 warped by sigma -> shift sigma / (1 + (shift - 1) sigma), the
    usual timestep shift of flow-matching video models."""
    s = np.linspace(1.0, 0.0, n + 1)
    return shift * s / (1.0 + (shift - 1.0) * s)


@pytest.mark.parametrize("n,shift,top", [(4, 3.0, 1.0), (4, 5.0, 0.999), (50, 3.0, 0.999), (8, 1.0, 1.0)])
def test_sampler_coefficients_reproduce_the_oracle_update(n, shift, top):
    """The host-side weights of step i, applied as rho x + A (c0 x0 + c1 x0_prev), give the
    oracle's DPM-Solver++ update for every step of a schedule."""
    sig = [float(np.float32(v)) for v in top * _shifted_sigmas(n, shift)]
    rng = np.random.default_rng(0)
    x, x0, x0p = rng.standard_normal(5), rng.standard_normal(5), rng.standard_normal(5)
    for i in range(n):
        for order in (1, 2):
            cf = B.chorus_sampler_coefficients(sig, i, order)
            got = cf.rho * x + cf.A * (cf.c0 * x0 + cf.c1 * x0p)
            if order == 2 and i > 0 and sig[i + 1] > 0:
                want = O.dpmpp_2m(x, x0, x0p, sig[i - 1], sig[i], sig[i + 1])
            else:
                want = O.dpmpp_first_order(x, x0, sig[i], sig[i + 1])
                assert cf.c0 == 1.0 and cf.c1 == 0.0
            np.testing.assert_allclose(got, want, rtol=0, atol=2e-6 * (1 + abs(cf.c0) + abs(cf.c1)))
            assert cf.sigma_s == np.float32(sig[i])
            assert abs(cf.c0 + cf.c1 - 1.0) < 1e-6      # the extrapolation weights sum to one
    lib = P.load()
    out = B.SamplerCoef()
    arr = lambda v: (C.c_float * len(v))(*v)
    assert lib.chorus_sampler_coefficients(None, 4, 0, 1, C.byref(out)) == B.E_ARG
    assert lib.chorus_sampler_coefficients(arr([1, .5, 0]), 2, 2, 1, C.byref(out)) == B.E_ARG      # i out of range
    assert lib.chorus_sampler_coefficients(arr([1, .5, 0]), 2, 0, 3, C.byref(out)) == B.E_ARG      # order
    assert lib.chorus_sampler_coefficients(arr([.5, .5, 0]), 2, 0, 1, C.byref(out)) == B.E_ARG     # not decreasing
    assert lib.chorus_sampler_coefficients(arr([.4, .5, .2]), 2, 1, 2, C.byref(out)) == B.E_ARG    # previous level below
    assert lib.chorus_sampler_coefficients(arr([1.5, .5, 0]), 2, 0, 1, C.byref(out)) == B.E_ARG    # above 1


def test_solver_entry_points_validate():
    lib = P.load()
    null, p16 = C.c_void_p(0), C.c_void_p(16)
    cf = B.SamplerCoef(0.5, 0.5, 0.5, 1.5, -0.5)
    gw = B.GlueWeights(16, 16, 16, 16, 16)
    args = lambda **k: [k.get("latent", p16), p16, null, 1.0, k.get("Ls", 4), null, C.byref(gw), p16, C.byref(cf),
                        k.get("x0_prev", C.c_void_p(32)), null, k.get("SL", null), k.get("mask", null), 64, 16, 1, 4, 4, 2,
                        2, k.get("ws", p16), k.get("ws_bytes", 1 << 30), null]
    assert lib.chorus_head_update_solver(*args(x0_prev=null)) == B.E_ARG          # second order without history
    assert lib.chorus_head_update_solver(*args(SL=C.c_void_p(48))) == B.E_ARG     # SL without mask
    assert lib.chorus_head_update_solver(*args(x0_prev=p16)) == B.E_ARG           # history aliases the latent
    assert lib.chorus_head_update_solver(*args(ws=null)) == B.E_WORKSPACE
    assert lib.chorus_head_update_solver(*args(ws_bytes=8)) == B.E_WORKSPACE
    assert lib.chorus_head_update_solver(*args(Ls=-1)) == B.E_ARG
    assert lib.chorus_head_update_solver(*args(Ls=0)) == B.OK
    assert lib.chorus_head_solver_workspace_bytes(64, 64, 100, 1) > lib.chorus_head_solver_workspace_bytes(64, 64, 100, 0)
    bs = B.make_block_shape(128, 2, 64, 256, 8, (1, 2, 2))
    ms = B.make_model_shape(bs, (16, 1, 4, 4), (2, 2), 1)
    a = lib.chorus_denoise_step_solver_workspace_bytes(C.byref(ms), 4, 0)
    b = lib.chorus_denoise_step_solver_workspace_bytes(C.byref(ms), 4, 1)
    assert 0 < a < b
    assert lib.chorus_denoise_run_workspace_bytes(C.byref(ms), 4) >= b


def test_head_update_region_validates():
    lib = P.load()
    null, p16 = C.c_void_p(0), C.c_void_p(16)
    gw = B.GlueWeights(16, 16, 16, 16, 16)
    args = lambda **k: [p16, p16, k.get("Ls", 4), null, C.byref(gw), p16, -0.25, k.get("SL", null), k.get("mask", null), 64, 16,
                        1, 4, 4, 2, 2, k.get("ws", p16), k.get("ws_bytes", 1 << 30), null]
    assert lib.chorus_head_update_region(*args(SL=C.c_void_p(48))) == B.E_ARG      # SL without mask
    assert lib.chorus_head_update_region(*args(mask=C.c_void_p(48))) == B.E_ARG    # mask without SL
    assert lib.chorus_head_update_region(*args(ws=null)) == B.E_WORKSPACE
    assert lib.chorus_head_update_region(*args(ws_bytes=8)) == B.E_WORKSPACE
    assert lib.chorus_head_update_region(*args(Ls=-1)) == B.E_ARG
    assert lib.chorus_head_update_region(*args(Ls=0)) == B.OK
    assert lib.chorus_head_update_region(*args(Ls=0, SL=C.c_void_p(48), mask=C.c_void_p(64))) == B.OK


def test_mfma_ceiling_validates():
    lib = P.load()
    out = C.c_double(0)
    need = lib.chorus_mfma_ceiling_workspace_bytes()
    assert need > 0
    assert lib.chorus_mfma_ceiling(1, 4, 1, C.byref(out), C.c_void_p(16), need, None) == B.E_ARG       # mix out of range
    assert lib.chorus_mfma_ceiling(1, 0, 0, C.byref(out), C.c_void_p(16), need, None) == B.E_ARG       # no launches
    assert lib.chorus_mfma_ceiling(1, 0, 1, None, C.c_void_p(16), need, None) == B.E_ARG
    assert lib.chorus_mfma_ceiling(1, 0, 1, C.byref(out), None, need, None) == B.E_WORKSPACE
    assert lib.chorus_mfma_ceiling(1, 0, 1, C.byref(out), C.c_void_p(16), need - 1, None) == B.E_WORKSPACE


@pytest.mark.parametrize("N", [4, 8, 50])
def test_schedule_with_stored_depths_matches_oracle(N):
    tau = 0.75
    for stored in ([1], [2], [3, 1], [N // 2, N // 4 + 1, N], list(range(1, N + 1)), []):
        for params in (None, dict(gamma_override=1.5), dict(a1=0.1, b1=0.5, a2=0.2, b2=0.3, r3=2)):
            for m in list(np.linspace(0.0, 1.0, 41)) + [float("nan")]:
                mf = float(np.float32(m))
                k1, k2, plan, slot = P.chorus_denoise_schedule(mf, tau, N, params, stored_steps=stored)
                ok1, ok2, oplan = O.denoise_schedule(mf, float(np.float32(tau)), N, params, stored_steps=stored)
                assert (k1, k2) == (ok1, ok2), (m, stored, params)
                assert slot == (stored.index(k1) if k1 > 0 else -1)
                for (s, gk, go), (os_, ogk, ogo) in zip(plan, oplan):
                    assert s == os_ and gk == np.float32(ogk) and go == np.float32(ogo)


def test_lookup_batch_validates():
    lib = P.load()
    null, p16 = C.c_void_p(0), C.c_void_p(16)
    need = lib.chorus_cache_lookup_batch_workspace_bytes(4096, 4096, 32)
    assert need > lib.chorus_cache_lookup_batch_workspace_bytes(4096, 4096, 16) > 0
    assert lib.chorus_cache_lookup_batch_workspace_bytes(-1, 8, 1) == 0
    call = lambda **k: lib.chorus_cache_lookup_batch(k.get("cache", p16), k.get("N", 8), k.get("d", 8), k.get("q", p16),
                                                      k.get("Q", 2), 0.5, k.get("k", 1), p16, p16, p16, k.get("ws", p16),
                                                      k.get("wsb", 1 << 30), null)
    assert call(d=6) == B.E_SHAPE
    assert call(k=0) == B.E_ARG and call(k=2000) == B.E_ARG
    assert call(N=-1) == B.E_ARG and call(q=null) == B.E_ARG and call(cache=null) == B.E_ARG
    assert call(cache=C.c_void_p(8)) == B.E_ARG                   # not 16-byte aligned
    assert call(ws=null) == B.E_WORKSPACE and call(wsb=16) == B.E_WORKSPACE
    assert call(Q=0) == B.OK


def test_time_mod_validates():
    lib = P.load()
    null, p16 = C.c_void_p(0), C.c_void_p(16)
    tw = B.TimeWeights(16, 16, 16, 16, 16, 16)
    need = lib.chorus_time_mod_workspace_bytes(256, 256)
    assert need > 0 and lib.chorus_time_mod_workspace_bytes(0, 256) == 0
    call = lambda **k: lib.chorus_time_mod(500.0, k.get("F", 256), k.get("D", 256), k.get("w", C.byref(tw)), k.get("tm", p16),
                                           p16, k.get("ws", p16), k.get("wsb", need), null)
    assert call(w=None) == B.E_ARG and call(tm=null) == B.E_ARG and call(D=0) == B.E_ARG
    assert call(F=12) == B.E_SHAPE and call(D=100) == B.E_SHAPE
    assert call(tm=C.c_void_p(4)) == B.E_ARG
    assert call(ws=null) == B.E_WORKSPACE and call(wsb=8) == B.E_WORKSPACE
    bad = B.TimeWeights(16, 16, 0, 16, 16, 16)
    assert call(w=C.byref(bad)) == B.E_ARG


def test_denoise_run_validates_before_any_launch():
    lib = P.load()
    bs = B.make_block_shape(128, 2, 64, 256, 8, (1, 2, 2))
    ms = B.make_model_shape(bs, (16, 1, 4, 4), (2, 2), 0)
    gw = B.GlueWeights(16, 16, 16, 16, 16)
    res = B.RunResult()
    sig = (C.c_float * 5)(1.0, 0.75, 0.5, 0.25, 0.0)
    need = lib.chorus_denoise_run_workspace_bytes(C.byref(ms), 4)
    assert need > 0

    def call(ws=C.c_void_p(256), wsb=None, **kw):
        f = dict(cache_emb=16, cache_latents=16, cache_N=4, cache_d=8, query=16, tau=0.75, sched=None, n_steps=4, sigmas=sig,
                 t_mods=16, t_heads=16, text_ctx=16, tdiff=0, mask_see=0, mask_edit=0, store_slot=-1, store_after=0,
                 latent_steps=None, n_latent_steps=0, solver_order=1, text_ctx_uncond=0, guidance=1.0)
        f.update(kw)
        rq = B.Request(**f)
        return lib.chorus_denoise_run(C.byref(ms), None, C.byref(gw), C.byref(rq), C.c_void_p(16), C.byref(res), ws,
                                      need if wsb is None else wsb, None)

    assert call(solver_order=3) == B.E_ARG and call(solver_order=-1) == B.E_ARG
    assert call(store_slot=4, store_after=1) == B.E_ARG                      # slot outside the cache
    assert call(store_slot=1, store_after=0) == B.E_ARG and call(store_slot=1, store_after=5) == B.E_ARG
    steps = lambda *v: (C.c_int32 * len(v))(*v)
    assert call(latent_steps=steps(1, 1), n_latent_steps=2) == B.E_ARG       # a depth listed twice
    assert call(latent_steps=steps(0), n_latent_steps=1) == B.E_ARG          # depth 0 is the noise itself
    assert call(latent_steps=steps(5), n_latent_steps=1) == B.E_ARG          # beyond the schedule
    assert call(latent_steps=steps(1), n_latent_steps=0) == B.E_ARG
    assert call(query=0) == B.E_ARG and call(sigmas=None) == B.E_ARG and call(n_steps=-1) == B.E_ARG
    assert call(ws=None) == B.E_WORKSPACE and call(wsb=need - 1) == B.E_WORKSPACE
    long_sig = (C.c_float * 66)(*[1.0 - i / 65 for i in range(66)])
    assert call(n_steps=65, sigmas=long_sig) == B.E_SHAPE                    # more steps than a plan holds: no launch
