"""GPU parity of the multistep sampler (DPM-Solver++ on the rectified-flow path), classifier-free
guidance and the latent fusion folded into the sampler pass, against the oracle."""
import numpy as np
import pytest
import torch

import synth
from oracle import chorus_oracle as O
import paper_2604_04451_amd as P
from paper_2604_04451_amd import binding as B
from gpu_util import DEV, check, dev_bf16, dev_f32, errs, host, host_bf16
from test_gpu_step import Model

pytestmark = pytest.mark.gpu


def _shifted(n, shift=3.0, top=1.0):
    s = np.linspace(1.0, 0.0, n + 1)
    return [float(np.float32(v)) for v in top * shift * s / (1.0 + (shift - 1.0) * s)]


def _uncond(md, seed=11):
    raw = synth.round_bf16(synth.normal(seed, "text_uncond", (md.bs.Lt, md.bs.text_dim), md.bs.text_std))
    d = B.chorus_text_project(dev_bf16(raw), md.dglue)
    return d, O.text_project(raw, md.gw)          # the oracle projects the prompt itself


def _u8(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint8)).to(DEV)


@pytest.mark.parametrize("cfg", [False, True])
def test_head_update_solver(cfg):
    print(f"[case] head_update_solver c1 cfg={cfg}", flush=True)
    bs = synth.SHAPES["c1"]
    md = Model(bs, 0)
    sig = _shifted(6)
    cf = B.chorus_sampler_coefficients(sig, 2, 2)
    assert cf.c1 != 0.0
    lat = synth.latent(bs, 0, std=1.0)
    x0p = synth.latent(bs, 0, "x0prev", std=1.0)
    SL = synth.latent(bs, 0, "SL", std=1.0)
    sel = synth.exact_count_mask(bs.L, 150, seed=3)
    idx = O.region_compact(sel)
    hist = synth.bernoulli_mask(bs.L, 0.5, seed=4)
    edit = (sel & synth.bernoulli_mask(bs.L, 0.6, seed=5)).astype(np.uint8)
    x = synth.normal(1, "hx", (idx.size, bs.D))
    xu = synth.normal(2, "hxu", (idx.size, bs.D))
    g = 3.0
    dl, dx0 = dev_f32(lat), dev_f32(x0p)
    B.chorus_head_update_solver(dl, dev_f32(x), idx.size, torch.from_numpy(idx.astype(np.int32)).to(DEV), md.dglue,
                                md.d_theads[0], cf, x0_prev=dx0, hist=_u8(hist), x_uncond=dev_f32(xu) if cfg else None,
                                guidance=g, SL=dev_f32(SL), mask_edit=_u8(edit))
    v = O.head(x, md.gw, md.t_heads[0])
    if cfg:
        v = O.cfg_combine(v, O.head(xu, md.gw, md.t_heads[0]), g)
    toks = O.patchify(lat.astype(np.float64), bs.patch)
    xs = toks[idx]
    x0 = O.velocity_to_x0(xs, v, sig[2])
    first = O.dpmpp_first_order(xs, x0, sig[2], sig[3])
    second = O.dpmpp_2m(xs, x0, O.patchify(x0p.astype(np.float64), bs.patch)[idx], sig[1], sig[2], sig[3])
    new = np.where((hist[idx] != 0)[:, None], second, first)
    sl_t = O.patchify(SL.astype(np.float64), bs.patch)[idx]
    new = np.where((edit[idx] != 0)[:, None], new, sl_t)
    ref = O.unpatchify(O.scatter_rows(toks, new, idx), lat.shape, bs.patch)
    ref_x0 = O.unpatchify(O.scatter_rows(O.patchify(x0p.astype(np.float64), bs.patch), x0, idx), lat.shape, bs.patch)
    # the head's velocity carries the bf16 rounding of its GEMM input (the same 8e-3 that the Euler test allows on v);
    # guidance combines two such velocities with weights g and g - 1
    tol = 8e-3 * ((2 * g - 1) if cfg else 1)
    check(host(dl), ref, "solver update latent", max_abs=tol, rel_l2=1e-3 * (3 if cfg else 1))
    check(host(dx0), ref_x0, "x0 history", max_abs=tol, rel_l2=1e-3 * (3 if cfg else 1))
    Ms = O.expand_token_mask(sel, bs.grid, bs.patch, bs.C).astype(bool)
    Mse = O.expand_token_mask(sel & (edit == 0), bs.grid, bs.patch, bs.C).astype(bool)
    np.testing.assert_array_equal(host(dl)[~Ms], lat[~Ms])              # tokens that are not selected: untouched
    np.testing.assert_array_equal(host(dx0)[~Ms], x0p[~Ms])
    np.testing.assert_array_equal(host(dl)[Mse], SL[Mse])               # selected, outside M_edit: the source latent
    # first-order weights: the Euler form of chorus_head_update, up to rounding
    cf1 = B.chorus_sampler_coefficients(sig, 2, 1)
    da, db = dev_f32(lat), dev_f32(lat)
    didx = torch.from_numpy(idx.astype(np.int32)).to(DEV)
    B.chorus_head_update_solver(da, dev_f32(x), idx.size, didx, md.dglue, md.d_theads[0], cf1)
    B.chorus_head_update(db, dev_f32(x), idx.size, didx, md.dglue, md.d_theads[0], sig[3] - sig[2])
    assert float((da - db).abs().max()) < 1e-5


@pytest.mark.parametrize("name,cfg", [("c1", False), ("c1", True), ("wan1p3b_small", False)])
def test_denoise_step_solver(name, cfg):
    print(f"[case] denoise_step_solver {name} cfg={cfg}", flush=True)
    bs = synth.SHAPES[name]
    md = Model(bs, 2, stress=(name == "c1"))
    sig = _shifted(6)
    lat = synth.latent(bs, 0, std=1.0)
    x0p = synth.latent(bs, 0, "x0prev", std=1.0)
    SL = synth.latent(bs, 0, "SL", std=1.0)
    kv = B.chorus_model_text_kv_project(md.model, md.arr, md.d_ctx)
    kvu, ctx_u, g = None, None, 1.0
    if cfg:
        d_ctx_u, ctx_u = _uncond(md)
        kvu, g = B.chorus_model_text_kv_project(md.model, md.arr, d_ctx_u), 3.0
    ks = synth.tdiff_scale(bs.Lt, 1.5)
    # stage 3, second order on a random half of the tokens
    hist = synth.bernoulli_mask(bs.L, 0.5, seed=4)
    cf = B.chorus_sampler_coefficients(sig, 2, 2)
    dl, dx0 = dev_f32(lat), dev_f32(x0p)
    B.chorus_denoise_step_solver(md.model, md.arr, md.dglue, dl, None, bs.L, kv, md.d_tmods[2], md.d_theads[2], cf,
                                 x0_prev=dx0, hist=_u8(hist), text_kv_uncond=kvu, guidance=g, tgaa_key_scale=dev_f32(ks),
                                 gamma_o=1.5)
    ref, ref_x0, _ = O.denoise_step_dpmpp(lat, md.blocks, md.gw, bs, md.ctx, md.t_mods[2], md.t_heads[2], sig[1], sig[2],
                                          sig[3], x0p, hist, text_ctx_uncond=ctx_u, guidance=g, key_scale=ks, gamma_o=1.5)
    check(host(dl), ref, "stage-3 solver step latent")
    check(host(dx0), ref_x0, "stage-3 solver step x0")
    a, r = errs(host(dl) - lat, ref - lat)
    print(f"[parity] stage-3 solver step update: rel_l2={r:.3e}", flush=True)
    assert r <= (6e-2 if cfg else 2e-2)
    # stage 2, M_edit strictly inside M_see, history on all tokens; the latent outside M_see is arbitrary, so Eq. 6 needs its pass
    T, Hg, Wg = bs.grid
    see = synth.box_mask(bs.grid, T, max(2, Hg * 2 // 3), max(2, Wg * 2 // 3), 0, 1, 1)
    edit = synth.box_mask(bs.grid, T, max(1, Hg * 2 // 3 - 2), max(1, Wg * 2 // 3 - 2), 0, 2, 2)
    idx_d, cnt = P.chorus_region_compact(_u8(see))
    Ls = int(cnt.cpu()[0])
    dl, dx0 = dev_f32(lat), dev_f32(x0p)
    B.chorus_denoise_step_solver(md.model, md.arr, md.dglue, dl, idx_d, Ls, kv, md.d_tmods[1], md.d_theads[1], cf,
                                 x0_prev=dx0, text_kv_uncond=kvu, guidance=g, tgaa_key_scale=dev_f32(ks), gamma_o=1.5,
                                 SL=dev_f32(SL), mask_edit=_u8(edit))
    ref, ref_x0, _ = O.denoise_step_dpmpp(lat, md.blocks, md.gw, bs, md.ctx, md.t_mods[1], md.t_heads[1], sig[1], sig[2],
                                          sig[3], x0p, np.ones(bs.L, np.uint8), text_ctx_uncond=ctx_u, guidance=g,
                                          mask_see=see, mask_edit=edit, SL=SL, key_scale=ks, gamma_o=1.5)
    check(host(dl), ref, "stage-2 solver step latent")
    check(host(dx0), ref_x0, "stage-2 solver step x0")
    Me = O.expand_token_mask(edit, bs.grid, bs.patch, bs.C).astype(bool)
    np.testing.assert_array_equal(host(dl)[~Me], SL[~Me])
    # the same step on a latent that already holds SL outside M_see, without the extra pass: same result bit for bit
    Ms = O.expand_token_mask(see, bs.grid, bs.patch, bs.C).astype(bool)
    lat2 = np.where(Ms, lat, SL).astype(np.float32)
    da, db = dev_f32(lat2), dev_f32(lat2)
    for d_, flag in ((da, False), (db, True)):
        B.chorus_denoise_step_solver(md.model, md.arr, md.dglue, d_, idx_d, Ls, kv, md.d_tmods[1], md.d_theads[1], cf,
                                     x0_prev=dev_f32(x0p), text_kv_uncond=kvu, guidance=g, tgaa_key_scale=dev_f32(ks),
                                     gamma_o=1.5, SL=dev_f32(SL), mask_edit=_u8(edit), outside_is_source=flag)
    assert torch.equal(da, db)
    check(host(db), ref, "stage-2 solver step latent, fusion inside the sampler pass")


@pytest.mark.parametrize("name,n_steps,cfg", [("c1", 4, False), ("c1", 8, True), ("wan1p3b_small", 4, False)])
def test_denoise_run_multistep(name, n_steps, cfg):
    """Hit (stage 1, stage 2 with M_edit inside M_see, stage 3) and miss with the second-order solver, with and
    without classifier-free guidance, against the oracle's loop."""
    print(f"[case] denoise_run multistep {name} steps={n_steps} cfg={cfg}", flush=True)
    bs = synth.SHAPES[name]
    md = Model(bs, 2, n_steps=n_steps)
    sig = _shifted(n_steps, top=0.999 if cfg else 1.0)
    N = 16
    cache = synth.cache_embeddings(N, bs.cache_d, seed=0)
    cache_lat = synth.normal(0, "cache_lat", (N,) + bs.latent_shape)
    noise = synth.latent(bs, 0, "noise", std=1.0)
    T, Hg, Wg = bs.grid
    see = synth.box_mask(bs.grid, T, Hg * 4 // 5, Wg // 2, 0, 1, 2)
    edit = synth.box_mask(bs.grid, T, Hg * 4 // 5 - 2, Wg // 2 - 2, 0, 2, 3)
    assert ((edit == 0) | (see == 1)).all() and 0 < edit.sum() < see.sum()
    tdiff = np.zeros(bs.Lt, np.uint8)
    tdiff[synth.stream(0, "tdiff").permutation(bs.Lt)[:max(1, bs.Lt // 64)]] = 1
    sched = dict(gamma_override=1.5)
    d_ctx_u, ctx_u, g = None, None, 1.0
    if cfg:
        (d_ctx_u, ctx_u), g = _uncond(md), 2.5
    ks_of = lambda gk: np.where(tdiff != 0, gk, 1.0)
    for near in (5, None):
        q = synth.cache_query(cache, seed=0, near=near)
        dl = dev_f32(noise)
        res = B.chorus_denoise_run(md.model, md.arr, md.dglue, dl, dev_f32(cache), dev_f32(cache_lat), dev_f32(q), 0.75,
                                   sig, md.d_tmods, md.d_theads, md.d_ctx, tdiff=_u8(tdiff), mask_see=_u8(see),
                                   mask_edit=_u8(edit), sched=sched, solver_order=2, text_ctx_uncond=d_ctx_u, guidance=g)
        oj, om, ohit = O.cache_lookup(cache, q, 0.75)
        K1, K2, plan = O.denoise_schedule(float(np.float32(res["score"])), float(np.float32(0.75)), n_steps, sched)
        assert (res["index"], res["hit"], res["K1"], res["K2"]) == (oj, ohit, K1, K2)
        stages = [p[0] for p in plan]
        if near is not None:
            assert ohit and 1 in stages and 2 in stages and stages.count(3) >= 2
        else:
            assert stages == [3] * n_steps
        ref = O.run_schedule_dpmpp(plan, sig, noise, cache_lat[oj], md.blocks, md.gw, bs, md.ctx, md.t_mods, md.t_heads,
                                   order=2, text_ctx_uncond=ctx_u, guidance=g, mask_see=see, mask_edit=edit,
                                   key_scale_of=ks_of)
        a_err, _ = check(host(dl), ref, f"multistep run near={near} latent")
        if near is None and not cfg:
            # the second-order term matters: the first-order run differs by far more than the parity tolerance
            ref1 = O.run_schedule_dpmpp(plan, sig, noise, cache_lat[oj], md.blocks, md.gw, bs, md.ctx, md.t_mods,
                                        md.t_heads, order=1)
            print(f"[info] order 2 vs order 1 run: max_abs={np.abs(ref - ref1).max():.3e}", flush=True)
            assert a_err < 0.25 * np.abs(ref - ref1).max()


def test_head_update_solver_full_shape_token_sampled():
    """The sampler pass at the 480p size (32760 tokens, 13104 selected, guidance on): the oracle evaluates a seeded
    sample of the selected tokens; every other cell is checked by what it must be bit for bit."""
    bs = synth.SHAPES["wan1p3b_480p"]
    print("[case] head_update_solver 1.3B 480p full shape", flush=True)
    gw = synth.glue_weights(bs, 0)
    dglue = B.upload_glue_weights(gw)
    t_head = synth.normal(0, "th", (2, bs.D), 0.02)
    sig = _shifted(4)
    cf = B.chorus_sampler_coefficients(sig, 2, 2)
    see = synth.box_mask(bs.grid, 21, 24, 26, 0, 3, 13)
    edit = synth.box_mask(bs.grid, 21, 22, 24, 0, 4, 14)
    hist = synth.bernoulli_mask(bs.L, 0.5, seed=4)
    idx = O.region_compact(see)
    lat = synth.latent(bs, 0, std=1.0)
    x0p = synth.latent(bs, 0, "x0prev", std=1.0)
    SL = synth.latent(bs, 0, "SL", std=1.0)
    x = synth.normal(1, "hx", (idx.size, bs.D)).astype(np.float32)
    xu = synth.normal(2, "hxu", (idx.size, bs.D)).astype(np.float32)
    g = 2.5
    dl, dx0 = dev_f32(lat), dev_f32(x0p)
    B.chorus_head_update_solver(dl, dev_f32(x), idx.size, torch.from_numpy(idx.astype(np.int32)).to(DEV), dglue,
                                dev_f32(t_head), cf, x0_prev=dx0, hist=_u8(hist), x_uncond=dev_f32(xu), guidance=g,
                                SL=dev_f32(SL), mask_edit=_u8(edit))
    got, got_x0 = host(dl), host(dx0)
    rows = np.unique(np.concatenate([synth.stream(5, "rows").permutation(idx.size)[:64], [0, idx.size - 1]]))
    tok = idx[rows]
    v = O.cfg_combine(O.head(x[rows], gw, t_head), O.head(xu[rows], gw, t_head), g)
    pick = lambda a: O.patchify(np.asarray(a, np.float64), bs.patch)[tok]
    xs = pick(lat)
    x0 = O.velocity_to_x0(xs, v, sig[2])
    new = np.where((hist[tok] != 0)[:, None], O.dpmpp_2m(xs, x0, pick(x0p), sig[1], sig[2], sig[3]),
                   O.dpmpp_first_order(xs, x0, sig[2], sig[3]))
    new = np.where((edit[tok] != 0)[:, None], new, pick(SL))
    check(pick(got), new, "full-shape solver update (sampled tokens)", max_abs=8e-3 * (2 * g - 1), rel_l2=3e-3)
    check(pick(got_x0), x0, "full-shape x0 history (sampled tokens)", max_abs=8e-3 * (2 * g - 1), rel_l2=3e-3)
    Ms = O.expand_token_mask(see, bs.grid, bs.patch, bs.C).astype(bool)
    Mse = O.expand_token_mask(see & (edit == 0), bs.grid, bs.patch, bs.C).astype(bool)
    np.testing.assert_array_equal(got[~Ms], lat[~Ms])
    np.testing.assert_array_equal(got_x0[~Ms], x0p[~Ms])
    np.testing.assert_array_equal(got[Mse], SL[Mse])
    Me = O.expand_token_mask(edit, bs.grid, bs.patch, bs.C).astype(bool)
    assert np.isfinite(got).all() and (got[Me] != lat[Me]).mean() > 0.99


def test_denoise_run_region_stage_first_and_fifty_steps():
    """Two schedules the 4-step default never produces: (a) a hit whose region stage starts at step 0 (no reused step
    before it, so Eq. 6 needs its own pass over the tokens outside M_see), Euler and multistep; (b) the 50-step
    configuration with guidance (threshold 0.65, Sec. 4.1 / Table 1) on the small model."""
    bs = synth.SHAPES["c1"]
    N = 16
    cache = synth.cache_embeddings(N, bs.cache_d, seed=0)
    cache_lat = synth.normal(0, "cache_lat", (N,) + bs.latent_shape)
    noise = synth.latent(bs, 0, "noise", std=1.0)
    T, Hg, Wg = bs.grid
    see = synth.box_mask(bs.grid, T, Hg * 4 // 5, Wg // 2, 0, 1, 2)
    edit = synth.box_mask(bs.grid, T, Hg * 4 // 5 - 2, Wg // 2 - 2, 0, 2, 3)
    q = synth.cache_query(cache, seed=0, near=5)
    ks_of = lambda gk: np.full(bs.Lt, gk)
    # (a)
    print("[case] denoise_run with the region stage at step 0 (c1)", flush=True)
    md = Model(bs, 2)
    sched = dict(a1=0.0, b1=0.0, a2=0.5, b2=0.0, gamma_override=1.5)
    for order in (1, 2):
        sig = md.sigmas if order == 1 else _shifted(4)
        dl = dev_f32(noise)
        res = B.chorus_denoise_run(md.model, md.arr, md.dglue, dl, dev_f32(cache), dev_f32(cache_lat), dev_f32(q), 0.75, sig,
                                   md.d_tmods, md.d_theads, md.d_ctx, mask_see=_u8(see), mask_edit=_u8(edit), sched=sched,
                                   solver_order=order)
        K1, K2, plan = O.denoise_schedule(float(np.float32(res["score"])), float(np.float32(0.75)), 4, sched)
        assert res["hit"] and (res["K1"], res["K2"]) == (K1, K2) == (0, 2)
        run = O.run_schedule if order == 1 else (lambda *a, **k: O.run_schedule_dpmpp(*a, order=2, **k))
        ref = run(plan, sig, noise, cache_lat[5], md.blocks, md.gw, bs, md.ctx, md.t_mods, md.t_heads, mask_see=see,
                  mask_edit=edit, key_scale_of=ks_of)
        check(host(dl), ref, f"region stage first, solver order {order}")
    # (b)
    print("[case] denoise_run 50 steps with guidance (c1)", flush=True)
    md = Model(bs, 2, n_steps=50)
    sig = _shifted(50, top=0.999)
    d_ctx_u, ctx_u = _uncond(md)
    dl = dev_f32(noise)
    res = B.chorus_denoise_run(md.model, md.arr, md.dglue, dl, dev_f32(cache), dev_f32(cache_lat), dev_f32(q), 0.65, sig,
                               md.d_tmods, md.d_theads, md.d_ctx, mask_see=_u8(see), mask_edit=_u8(edit), solver_order=2,
                               text_ctx_uncond=d_ctx_u, guidance=2.0)
    K1, K2, plan = O.denoise_schedule(float(np.float32(res["score"])), float(np.float32(0.65)), 50)
    assert res["hit"] and (res["K1"], res["K2"]) == (K1, K2) and 1 <= K1 < K2 < 50
    print(f"[info] 50-step plan: K1={K1} K2={K2}", flush=True)
    ref = O.run_schedule_dpmpp(plan, sig, noise, cache_lat[5], md.blocks, md.gw, bs, md.ctx, md.t_mods, md.t_heads, order=2,
                               text_ctx_uncond=ctx_u, guidance=2.0, mask_see=see, mask_edit=edit,
                               key_scale_of=lambda gk: np.full(bs.Lt, gk))
    check(host(dl), ref, "50-step run with guidance")
