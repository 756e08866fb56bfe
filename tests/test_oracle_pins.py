"""Pins for the CPU oracle: every function is checked against something other than
itself -- brute force in pure Python on tiny inputs, closed forms, invariants the
paper states, and torch-CPU library routines as a third opinion. CPU only."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as TF

import synth
from oracle import chorus_oracle as O

T64 = torch.float64


# ------------------------------------------------------------------ lookup

def _brute_lookup(cache, q):
    best, bj = -math.inf, -1
    nq = math.sqrt(sum(float(a) * float(a) for a in q))
    for j, row in enumerate(cache):
        d = sum(float(a) * float(b) for a, b in zip(row, q))
        nc = math.sqrt(sum(float(a) * float(a) for a in row))
        s = d / (nq * nc) if nq * nc > 0 else -math.inf
        if s > best:
            best, bj = s, j
    return bj, best


def test_lookup_brute_force():
    cache = synth.cache_embeddings(8, 256, seed=0)
    q = synth.cache_query(cache, seed=0, near=5)
    j, m, hit = O.cache_lookup(cache, q, 0.75)
    bj, bm = _brute_lookup(cache, q)
    assert j == bj == 5
    assert abs(m - bm) < 1e-12
    assert hit == (bm >= 0.75)


def test_lookup_self_query_and_numpy_argmax():
    cache = synth.cache_embeddings(64, 128, seed=1)
    for j in (0, 17, 63):
        jj, m, hit = O.cache_lookup(cache, cache[j], 0.75)
        assert jj == j and abs(m - 1.0) < 1e-6 and hit
    q = synth.cache_query(cache, seed=1, near=None)
    jj, m, hit = O.cache_lookup(cache, q, 0.75)
    # rows are unit norm, so cosine ranking == dot ranking
    assert jj == int(np.argmax(cache.astype(np.float64) @ q.astype(np.float64)))
    assert not hit  # uniform query in 128-d: cosine far below 0.75


def test_lookup_scale_invariance_and_non_unit_rows():
    # cosine, not dot: a long row must not win on length alone
    cache = np.array([[10.0, 10.0], [1.0, 0.0], [0.0, 3.0]], np.float32)
    j, m, _ = O.cache_lookup(cache, np.array([2.0, 0.1], np.float32), 0.5)
    assert j == 1
    j2, m2, _ = O.cache_lookup(cache * 8.0, np.array([2.0, 0.1], np.float32) * 0.25, 0.5)
    assert j2 == 1 and abs(m - m2) < 1e-12


def test_lookup_ties_empty_single_zero_norm():
    cache = synth.cache_embeddings(16, 32, seed=2)
    cache[11] = cache[3]
    j, m, _ = O.cache_lookup(cache, cache[3], 0.75)
    assert j == 3  # lowest index among equal maxima
    assert O.cache_lookup(np.zeros((0, 32), np.float32), cache[0], 0.75) == (-1, -math.inf, False)
    j, m, hit = O.cache_lookup(cache[:1], cache[0], 0.75)
    assert j == 0 and hit
    z = cache.copy()
    z[0] = 0
    s = O.cosine_scores(z, cache[1])
    assert s[0] == -math.inf and np.isfinite(s[1:]).all()
    j, m, hit = O.cache_lookup(cache, np.zeros(32, np.float32), 0.75)
    assert m == -math.inf and not hit


def test_lookup_threshold_is_inclusive():
    # Sec. 3.1: the miss condition is m < tau, so m == tau is a hit
    cache = np.array([[1.0, 0.0], [0.0, 1.0]], np.float32)
    j, m, hit = O.cache_lookup(cache, np.array([1.0, 0.0], np.float32), 1.0)
    assert (j, m, hit) == (0, 1.0, True)


# ---------------------------------------------------------------- schedule

@pytest.mark.parametrize("N", [1, 4, 8, 50])
@pytest.mark.parametrize("tau", [0.65, 0.75])
def test_schedule_properties(N, tau):
    prev = (0, 0)
    prev_first_gamma = None
    for m in np.linspace(0.0, 1.0, 201):
        K1, K2, plan = O.denoise_schedule(float(m), tau, N)
        assert len(plan) == N
        assert 0 <= K1 <= K2 <= N                      # Eq. 1 bounds
        if m < tau:
            assert (K1, K2) == (0, 0)                  # fallback rule
            assert all(p == (3, 1.0, 1.0) for p in plan)
            continue
        assert K1 >= prev[0] and K2 >= prev[1]         # monotone in m
        prev = (K1, K2)
        stages = [p[0] for p in plan]
        assert stages == [1] * K1 + [2] * (K2 - K1) + [3] * (N - K2)
        assert K2 <= N - 1 or N == 0                   # at least one full-compute step
        gk = [p[1] for p in plan[K1:]]
        go = [p[2] for p in plan[K1:]]
        assert all(g >= 1.0 for g in gk + go)          # clamp
        assert all(a >= b for a, b in zip(gk, gk[1:]))  # decreasing with the step
        assert all(a >= b for a, b in zip(go, go[1:]))
        if gk:
            if prev_first_gamma is not None:
                assert gk[0] <= prev_first_gamma + 1e-12  # decreasing with m
            prev_first_gamma = gk[0]


def test_schedule_four_step_plan_and_override():
    K1, K2, plan = O.denoise_schedule(0.8, 0.75, 4)
    assert (K1, K2) == (1, 2) and [p[0] for p in plan] == [1, 2, 3, 3]
    assert plan[1][1] > 1.0 and plan[2][1:] == (1.0, 1.0) and plan[3][1:] == (1.0, 1.0)
    _, _, plan = O.denoise_schedule(0.8, 0.75, 4, dict(gamma_override=1.5))
    assert plan[1] == (2, 1.5, 1.5)
    # NaN / -inf scores (empty cache) fall back to plain generation
    assert O.denoise_schedule(-math.inf, 0.75, 4)[:2] == (0, 0)
    assert O.denoise_schedule(float("nan"), 0.75, 4)[:2] == (0, 0)


# ------------------------------------------------- pointwise vs torch / closed forms

def test_layernorm_rms_gelu_linear_vs_torch():
    x = synth.normal(3, "p.x", (37, 96), 1.7, 0.3).astype(np.float64)
    xt = torch.from_numpy(x)
    np.testing.assert_allclose(O.layernorm(x), TF.layer_norm(xt, (96,), eps=1e-6).numpy(), rtol=0, atol=1e-12)
    ln = O.layernorm(x)
    assert np.abs(ln.mean(-1)).max() < 1e-12 and np.abs(ln.var(-1) - 1).max() < 1e-5
    g = synth.normal(3, "p.g", (96,), 0.2, 1.0).astype(np.float64)
    np.testing.assert_allclose(O.rmsnorm(x, g), TF.rms_norm(xt, (96,), torch.from_numpy(g), eps=1e-6).numpy(),
                               rtol=0, atol=1e-12)
    r = O.rmsnorm(x * 100, np.ones(96))
    np.testing.assert_allclose(np.sqrt((r * r).mean(-1)), 1.0, atol=1e-8)
    np.testing.assert_allclose(O.gelu_tanh(x), TF.gelu(xt, approximate="tanh").numpy(), rtol=0, atol=1e-14)
    assert abs(float(O.gelu_tanh(np.array(0.0)))) == 0.0 and abs(float(O.gelu_tanh(np.array(10.0))) - 10.0) < 1e-9
    w = synth.normal(3, "p.w", (40, 96)).astype(np.float64)
    b = synth.normal(3, "p.b", (40,)).astype(np.float64)
    np.testing.assert_allclose(O.linear(x, w, b), TF.linear(xt, torch.from_numpy(w), torch.from_numpy(b)).numpy(),
                               rtol=0, atol=1e-11)
    # triple loop on a corner
    y = O.linear(x, w, b)
    for i, j in ((0, 0), (36, 39), (5, 17)):
        assert abs(y[i, j] - (sum(x[i, k] * w[j, k] for k in range(96)) + b[j])) < 1e-11


def _rope_complex(z, token_idx, grid, H, dh, theta=10000.0):
    """Independent formulation: each (even, odd) pair is a complex number multiplied by e^{i pos w}."""
    L = z.shape[0]
    zc = z.reshape(L, H, dh // 2, 2)
    zc = zc[..., 0] + 1j * zc[..., 1]
    T, Hg, Wg = grid
    n = np.asarray(token_idx)
    coords = (n // (Hg * Wg), (n // Wg) % Hg, n % Wg)
    s = dh // 6
    sizes = (dh - 4 * s, 2 * s, 2 * s)
    freqs = []
    for g, c in zip(sizes, coords):
        inv = theta ** (-np.arange(0, g, 2, dtype=np.float64) / g)
        freqs.append(np.exp(1j * c[:, None].astype(np.float64) * inv[None]))
    rot = np.concatenate(freqs, axis=1)  # [L, dh/2]
    out = zc * rot[:, None, :]
    return np.stack([out.real, out.imag], -1).reshape(L, H * dh)


@pytest.mark.parametrize("dh,H", [(64, 4), (128, 2)])
def test_rope(dh, H):
    assert O.rope_group_sizes(128) == (44, 42, 42) and O.rope_group_sizes(64) == (24, 20, 20)
    grid = (4, 6, 5)
    L = 4 * 6 * 5
    z = synth.normal(4, f"rope{dh}", (L, H * dh)).astype(np.float64)
    idx = np.arange(L)
    r = O.rope3d(z, idx, grid, H, dh)
    np.testing.assert_allclose(r, _rope_complex(z, idx, grid, H, dh), atol=1e-12)
    np.testing.assert_array_equal(r[0], z[0])                      # position (0,0,0) is the identity
    np.testing.assert_allclose((r * r).sum(-1), (z * z).sum(-1), rtol=1e-12)  # rotation keeps norms
    # relative-position property: <R(p) q, R(p') k> depends only on p - p'
    q = z[7:8].repeat(L, 0)
    k = z[9:10].repeat(L, 0)
    rq, rk = O.rope3d(q, idx, grid, H, dh), O.rope3d(k, idx, grid, H, dh)
    pos = np.stack(O.token_positions(idx, grid), -1)
    ix = lambda t, h, w: (t * 6 + h) * 5 + w
    a, b, c, d = ix(1, 2, 1), ix(2, 4, 3), ix(2, 3, 2), ix(3, 5, 4)   # b - a == d - c == (1, 2, 2)
    assert ((pos[b] - pos[a]) == (pos[d] - pos[c])).all()
    for hh in range(H):
        sl = slice(hh * dh, (hh + 1) * dh)
        assert abs(rq[a, sl] @ rk[b, sl] - rq[c, sl] @ rk[d, sl]) < 1e-10
        assert abs(rq[a, sl] @ rk[b, sl] - rq[a, sl] @ rk[d, sl]) > 1e-6   # and does depend on the offset
    # compacted subset keeps original positions
    sub = np.array([3, 50, 51, 119])
    np.testing.assert_array_equal(O.rope3d(z[sub], sub, grid, H, dh), r[sub])


def test_token_positions():
    t, h, w = O.token_positions(np.array([0, 1, 52, 30 * 52, 21 * 30 * 52 - 1]), (21, 30, 52))
    assert list(t) == [0, 0, 0, 1, 20] and list(h) == [0, 0, 1, 0, 29] and list(w) == [0, 1, 0, 0, 51]


# --------------------------------------------------------------- attention

def _brute_attention(q, k, v, H, dh):
    Lq, Lk = q.shape[0], k.shape[0]
    out = np.zeros((Lq, H * dh))
    for h in range(H):
        for i in range(Lq):
            logits = [sum(q[i, h * dh + c] * k[j, h * dh + c] for c in range(dh)) / math.sqrt(dh) for j in range(Lk)]
            mx = max(logits)
            e = [math.exp(l - mx) for l in logits]
            s = sum(e)
            for c in range(dh):
                out[i, h * dh + c] = sum(e[j] / s * v[j, h * dh + c] for j in range(Lk))
    return out


def test_attention_brute_force_and_sdpa():
    H, dh, Lq, Lk = 2, 8, 5, 7
    q = synth.normal(5, "a.q", (Lq, H * dh), 2.0).astype(np.float64)
    k = synth.normal(5, "a.k", (Lk, H * dh), 2.0).astype(np.float64)
    v = synth.normal(5, "a.v", (Lk, H * dh)).astype(np.float64)
    o, probs = O.attention(q, k, v, H, dh, return_probs=True)
    np.testing.assert_allclose(o, _brute_attention(q, k, v, H, dh), atol=1e-12)
    for p in probs:
        np.testing.assert_allclose(p.sum(-1), 1.0, atol=1e-14)   # rows sum to 1
    tq, tk, tv = (torch.from_numpy(a).reshape(-1, H, dh).transpose(0, 1) for a in (q, k, v))
    ref = TF.scaled_dot_product_attention(tq, tk, tv).transpose(0, 1).reshape(Lq, H * dh).numpy()
    np.testing.assert_allclose(o, ref, atol=1e-12)


def test_attention_closed_forms():
    H, dh, Lq, Lk = 3, 4, 6, 9
    v = synth.normal(6, "c.v", (Lk, H * dh)).astype(np.float64)
    q = synth.normal(6, "c.q", (Lq, H * dh)).astype(np.float64)
    # equal logits -> mean of V
    o = O.attention(q, np.zeros((Lk, H * dh)), v, H, dh)
    np.testing.assert_allclose(o, np.broadcast_to(v.mean(0), o.shape), atol=1e-14)
    # one key -> V
    o = O.attention(q, q[:1], v[:1], H, dh)
    np.testing.assert_allclose(o, np.broadcast_to(v[0], o.shape), atol=1e-14)
    # a dominating key -> its V
    k = np.zeros((Lk, H * dh))
    k[4] = 1e3 * np.sign(q[2])
    o = O.attention(q[2:3], k, v, H, dh)
    np.testing.assert_allclose(o[0], v[4], atol=1e-9)


# ------------------------------------------------------------------- TGAA

def _cross_inputs(seed=7, Lq=10, Lt=6, H=2, dh=8):
    q = synth.normal(seed, "t.q", (Lq, H * dh), 1.5).astype(np.float64)
    k = synth.normal(seed, "t.k", (Lt, H * dh), 1.5).astype(np.float64)
    v = synth.normal(seed, "t.v", (Lt, H * dh)).astype(np.float64)
    return q, k, v, H, dh


def test_tgaa_key_amplification():
    q, k, v, H, dh = _cross_inputs()
    plain = O.attention(q, k, v, H, dh)
    # neutral amplification is plain cross-attention, bit for bit
    np.testing.assert_array_equal(O.attention(q, O.tgaa_amplify_keys(k, np.ones(6)), v, H, dh), plain)
    np.testing.assert_array_equal(O.attention(q, O.tgaa_amplify_keys(k, None), v, H, dh), plain)
    # g == c on all tokens is attention with softmax scale c/sqrt(dh)
    tq, tk, tv = (torch.from_numpy(a).reshape(-1, H, dh).transpose(0, 1) for a in (q, k, v))
    ref = TF.scaled_dot_product_attention(tq, tk, tv, scale=1.5 / math.sqrt(dh)).transpose(0, 1).reshape(10, H * dh)
    np.testing.assert_allclose(O.attention(q, O.tgaa_amplify_keys(k, np.full(6, 1.5)), v, H, dh), ref.numpy(), atol=1e-12)
    # Eq. 2 on a strict subset: scaled key rows == per-column logit scale
    g = np.ones(6)
    g[[1, 4]] = 1.5
    amp = O.attention(q, O.tgaa_amplify_keys(k, g), v, H, dh)
    for h in range(H):
        sl = slice(h * dh, (h + 1) * dh)
        logits = (q[:, sl] @ k[:, sl].T) / math.sqrt(dh) * g[None, :]
        p = np.exp(logits - logits.max(-1, keepdims=True))
        p /= p.sum(-1, keepdims=True)
        np.testing.assert_allclose(amp[:, sl], p @ v[:, sl], atol=1e-12)
    # only the selected rows of K change
    kp = O.tgaa_amplify_keys(k, g)
    np.testing.assert_array_equal(kp[[0, 2, 3, 5]], k[[0, 2, 3, 5]])
    np.testing.assert_array_equal(kp[[1, 4]], 1.5 * k[[1, 4]])
    assert np.abs(amp - plain).max() > 1e-3


# ------------------------------------------------------------------ block

class _Shape:
    def __init__(self, D, H, dh, grid):
        self.D, self.H, self.dh, self.grid = D, H, dh, grid


def _small_block(seed=0, stress=True, D=48, H=2, dh=24, F=80, Lt=5, grid=(2, 3, 4)):
    bs = synth.BlockShape("t", D=D, H=H, dh=dh, F=F, Lt=Lt, text_dim=D, grid=grid)
    w = synth.stress_block_weights(bs, seed) if stress else synth.block_weights(bs, seed)
    inp = synth.block_inputs(bs, seed, x_std=1.0)
    return bs, w, inp


def _torch_block(x, w, bs, ctx, t_mod, token_idx, key_scale, gamma_o, key_mask=None):
    """Third opinion: the same block composed from torch-CPU library routines in fp64
    (layer_norm, rms_norm, linear, gelu, scaled_dot_product_attention) with the
    complex-number RoPE above. key_mask (bool [L]) runs the DENSE masked form:
    all tokens are queries, keys outside the mask get -inf."""
    D, H, dh = bs.D, bs.H, bs.dh
    t = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    x = t(x)
    e = t(w["mod_table"]) + t(t_mod)
    sh1, sc1, g1, sh2, sc2, g2 = e
    h = TF.layer_norm(x, (D,), eps=1e-6) * (1 + sc1) + sh1
    qkv = TF.linear(h, t(w["w_qkv"]), t(w["b_qkv"]))
    q, k, v = qkv[:, :D], qkv[:, D:2 * D], qkv[:, 2 * D:]
    q = TF.rms_norm(q, (D,), t(w["g_q"]), eps=1e-6)
    k = TF.rms_norm(k, (D,), t(w["g_k"]), eps=1e-6)
    q = t(_rope_complex(q.numpy(), token_idx, bs.grid, H, dh))
    k = t(_rope_complex(k.numpy(), token_idx, bs.grid, H, dh))
    sp = lambda a: a.reshape(-1, H, dh).transpose(0, 1)
    am = None
    if key_mask is not None:
        am = torch.zeros(x.shape[0], x.shape[0], dtype=T64)
        am[:, ~torch.from_numpy(key_mask)] = -math.inf
    o = TF.scaled_dot_product_attention(sp(q), sp(k), sp(v), attn_mask=am).transpose(0, 1).reshape(-1, D)
    x = x + g1 * TF.linear(o, t(w["w_o"]), t(w["b_o"]))
    hc = TF.layer_norm(x, (D,), t(w["ln3_w"]), t(w["ln3_b"]), eps=1e-6)
    qc = TF.rms_norm(TF.linear(hc, t(w["w_cq"]), t(w["b_cq"])), (D,), t(w["g_cq"]), eps=1e-6)
    kv = TF.linear(t(ctx), t(w["w_ckv"]), t(w["b_ckv"]))
    kc = TF.rms_norm(kv[:, :D], (D,), t(w["g_ck"]), eps=1e-6)
    vc = kv[:, D:]
    if key_scale is not None:
        kc = kc * t(key_scale)[:, None]
    oc = TF.scaled_dot_product_attention(sp(qc), sp(kc), sp(vc)).transpose(0, 1).reshape(-1, D)
    x = x + gamma_o * TF.linear(oc, t(w["w_co"]), t(w["b_co"]))
    h2 = TF.layer_norm(x, (D,), eps=1e-6) * (1 + sc2) + sh2
    y = TF.linear(TF.gelu(TF.linear(h2, t(w["w_1"]), t(w["b_1"])), approximate="tanh"), t(w["w_2"]), t(w["b_2"]))
    return (x + g2 * y).numpy()


def test_block_vs_torch_composition():
    bs, w, inp = _small_block()
    g = np.array([1.0, 1.5, 1.0, 1.5, 1.0])
    out = O.dit_block(inp["x"], w, bs, inp["text_ctx"], inp["t_mod"], key_scale=g, gamma_o=1.3)
    ref = _torch_block(inp["x"], w, bs, inp["text_ctx"], inp["t_mod"], np.arange(bs.L), g, 1.3)
    np.testing.assert_allclose(out, ref, atol=1e-10)
    assert np.abs(out - inp["x"]).max() > 0.1  # the branches are not negligible in this variant


def test_block_zero_gates_is_identity_and_gamma_o_linear():
    bs, w, inp = _small_block()
    w0 = dict(w)
    mt = w["mod_table"].copy()
    mt[2] = -inp["t_mod"][2]
    mt[5] = -inp["t_mod"][5]
    w0["mod_table"] = mt
    out = O.dit_block(inp["x"], w0, bs, inp["text_ctx"], inp["t_mod"], gamma_o=0.0)
    np.testing.assert_array_equal(out, inp["x"].astype(np.float64))
    # Eq. 3: with the FFN gate closed, x_out - x_in is affine in gamma_o with slope cross_attn(x)
    outs = [O.dit_block(inp["x"], w0, bs, inp["text_ctx"], inp["t_mod"], gamma_o=g) for g in (0.0, 1.0, 2.0)]
    np.testing.assert_allclose(outs[2] - outs[1], outs[1] - outs[0], atol=1e-12)
    _, br = O.dit_block(inp["x"], w0, bs, inp["text_ctx"], inp["t_mod"], gamma_o=1.0, return_branches=True)
    np.testing.assert_allclose(outs[1] - outs[0], br["y_ca"], atol=1e-12)


def test_block_neutral_tgaa_is_plain():
    bs, w, inp = _small_block(seed=1)
    a = O.dit_block(inp["x"], w, bs, inp["text_ctx"], inp["t_mod"])
    b = O.dit_block(inp["x"], w, bs, inp["text_ctx"], inp["t_mod"], key_scale=np.ones(bs.Lt), gamma_o=1.0)
    np.testing.assert_array_equal(a, b)


def test_block_row_subset_equals_full():
    bs, w, inp = _small_block(seed=2)
    full = O.dit_block(inp["x"], w, bs, inp["text_ctx"], inp["t_mod"], gamma_o=1.5)
    rows = np.array([0, 5, 6, 23])
    sub = O.dit_block(inp["x"], w, bs, inp["text_ctx"], inp["t_mod"], gamma_o=1.5, rows=rows)
    np.testing.assert_allclose(sub, full[rows], atol=1e-12)


def test_compacted_block_equals_dense_masked():
    """Sec. 3.3.3: selecting the region gives what a mask that merely removes the
    other tokens from attention would give, on the selected rows."""
    bs, w, inp = _small_block(seed=3)
    mask = synth.exact_count_mask(bs.L, 11, seed=3)
    idx = O.region_compact(mask)
    assert list(idx) == sorted(idx) and len(idx) == 11 and (mask[idx] == 1).all()
    comp = O.dit_block(inp["x"][idx], w, bs, inp["text_ctx"], inp["t_mod"], token_idx=idx, gamma_o=1.2)
    dense = _torch_block(inp["x"], w, bs, inp["text_ctx"], inp["t_mod"], np.arange(bs.L), None, 1.2,
                         key_mask=mask.astype(bool))
    np.testing.assert_allclose(comp, dense[idx], atol=1e-10)
    # all-ones mask is the unmasked block
    allm = np.ones(bs.L, np.uint8)
    np.testing.assert_array_equal(O.region_compact(allm), np.arange(bs.L))
    a = O.dit_block(inp["x"], w, bs, inp["text_ctx"], inp["t_mod"], token_idx=O.region_compact(allm))
    b = O.dit_block(inp["x"], w, bs, inp["text_ctx"], inp["t_mod"])
    np.testing.assert_array_equal(a, b)


# ------------------------------------------------------ gather / scatter / blend

def test_gather_scatter_roundtrip():
    x = synth.normal(8, "g.x", (20, 6))
    mask = synth.exact_count_mask(20, 7, seed=8)
    idx = O.region_compact(mask)
    g = O.gather_rows(x, idx)
    assert g.shape == (7, 6)
    for i, n in enumerate(idx):
        np.testing.assert_array_equal(g[i], x[n])
    y = O.scatter_rows(np.zeros_like(x), g, idx)
    np.testing.assert_array_equal(y[idx], x[idx])
    assert (y[mask == 0] == 0).all()
    assert O.region_compact(np.zeros(5, np.uint8)).size == 0


def test_blend_ends_and_select_form():
    grid, patch = (2, 3, 4), (1, 2, 2)
    shp = (3, 2, 6, 8)
    L = synth.normal(9, "b.L", shp)
    SL = synth.normal(9, "b.SL", shp)
    ones, zeros = np.ones(24, np.uint8), np.zeros(24, np.uint8)
    out = O.region_blend(L, SL, zeros, grid, patch)
    assert out.dtype == np.float32 and out.tobytes() == SL.tobytes()   # all-reuse: cached latent bit for bit
    assert O.region_blend(L, SL, ones, grid, patch).tobytes() == L.tobytes()  # all-compute
    m = synth.exact_count_mask(24, 9, seed=9)
    out = O.region_blend(L, SL, m, grid, patch)
    # explicit index loop (select form)
    for c in range(3):
        for t in range(2):
            for y in range(6):
                for x in range(8):
                    tok = (t * 3 + y // 2) * 4 + x // 2
                    assert out[c, t, y, x] == (L if m[tok] else SL)[c, t, y, x]


def test_patchify_roundtrip_and_layout():
    shp, patch = (3, 2, 4, 6), (1, 2, 2)
    lat = np.arange(np.prod(shp), dtype=np.float64).reshape(shp)
    tok = O.patchify(lat, patch)
    assert tok.shape == (2 * 2 * 3, 12)
    # token (t=1, hg=1, wg=2), feature (c=2, dy=1, dx=0)
    n = (1 * 2 + 1) * 3 + 2
    f = (2 * 1 + 0) * 4 + 1 * 2 + 0
    assert tok[n, f] == lat[2, 1, 1 * 2 + 1, 2 * 2 + 0]
    np.testing.assert_array_equal(O.unpatchify(tok, shp, patch), lat)


# -------------------------------------------------- model input / output stand-ins

def _loop_linear(x, w, b):
    """y[i][o] = sum_k x[i][k] * w[o][k] + b[o], written out."""
    return [[sum(float(xi[k]) * float(w[o][k]) for k in range(len(xi))) + float(b[o]) for o in range(len(w))] for xi in x]


def _loop_gelu_tanh(v):
    return 0.5 * v * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (v + 0.044715 * v ** 3)))


def test_patch_embed_text_project_head_written_out():
    """The model's input and output layers are stand-ins the paper does not define (Sec. 2.1 names the parts of a
    DiT only), so the only pin available is the definition written out as Python loops on a tiny case: the patch
    embedding (a linear map of the (c, dy, dx) cell), the text projection (linear, tanh-GELU, linear, in that
    order) and the head (LayerNorm without affine, times (1 + scale), plus shift, then linear; row 0 of the table
    is the shift, row 1 the scale). Biases and both modulation rows are non-zero and distinct, so a dropped bias,
    swapped layers, a swapped (shift, scale) pair or a missing "1 +" each fail."""
    rng = synth.stream(21, "glue-pin")
    D, P, Lt, Td, L = 6, 4, 3, 5, 4
    gw = {
        "w_patch": rng.normal(size=(D, P)), "b_patch": rng.normal(size=D),
        "w_text1": rng.normal(size=(D, Td)), "b_text1": rng.normal(size=D),
        "w_text2": rng.normal(size=(D, D)), "b_text2": rng.normal(size=D),
        "w_head": rng.normal(size=(P, D)), "b_head": rng.normal(size=P),
        "head_table": rng.normal(size=(2, D)),
    }
    # patch embedding
    patches = rng.normal(size=(L, P))
    np.testing.assert_allclose(O.patch_embed(patches, gw), _loop_linear(patches, gw["w_patch"], gw["b_patch"]), rtol=1e-12, atol=1e-12)
    # text projection
    text = rng.normal(size=(Lt, Td))
    hid = [[_loop_gelu_tanh(v) for v in row] for row in _loop_linear(text, gw["w_text1"], gw["b_text1"])]
    np.testing.assert_allclose(O.text_project(text, gw), _loop_linear(hid, gw["w_text2"], gw["b_text2"]), rtol=1e-12, atol=1e-12)
    # head
    x = rng.normal(size=(L, D)) * 2.0 + 0.5
    t_head = rng.normal(size=(2, D))
    mod = []
    for row in x:
        mu = sum(float(v) for v in row) / D
        var = sum((float(v) - mu) ** 2 for v in row) / D
        mod.append([(float(row[i]) - mu) / math.sqrt(var + 1e-6) * (1.0 + float(gw["head_table"][1][i]) + float(t_head[1][i]))
                    + float(gw["head_table"][0][i]) + float(t_head[0][i]) for i in range(D)])
    ref = np.array(_loop_linear(mod, gw["w_head"], gw["b_head"]))
    np.testing.assert_allclose(O.head(x, gw, t_head), ref, rtol=1e-12, atol=1e-12)
    # the planted mistakes are all visible at this size
    swapped = dict(gw, head_table=gw["head_table"][::-1].copy())
    assert np.abs(O.head(x, swapped, t_head[::-1]) - ref).max() > 1e-2
    # torch as a third opinion on the head's normalisation
    tx = torch.tensor(x, dtype=T64)
    tref = TF.linear(TF.layer_norm(tx, (D,), eps=1e-6) * (1.0 + torch.tensor(gw["head_table"][1] + t_head[1]))
                     + torch.tensor(gw["head_table"][0] + t_head[0]), torch.tensor(gw["w_head"]), torch.tensor(gw["b_head"]))
    np.testing.assert_allclose(O.head(x, gw, t_head), tref.numpy(), rtol=1e-12, atol=1e-12)


def test_step_euler_update_written_out():
    """One stage-3 step of a model without blocks is patchify -> embed -> head -> x + dsigma * v -> unpatchify:
    checked cell by cell with the written-out layers above, so the token / feature order of the update is pinned."""
    rng = synth.stream(22, "step-pin")
    bs = synth.BlockShape("pin", D=8, H=1, dh=8, F=8, Lt=2, text_dim=4, grid=(2, 2, 2), C=2)
    gw = synth.glue_weights(bs, 3, std=0.3)
    gw["b_patch"] = rng.normal(size=bs.D)
    gw["b_head"] = rng.normal(size=bs.patch_dim)
    lat = rng.normal(size=bs.latent_shape)
    t_head = rng.normal(size=(2, bs.D)) * 0.3
    out = O.denoise_step(lat, [], gw, bs, np.zeros((bs.Lt, bs.D)), np.zeros((6, bs.D)), t_head, -0.5)
    C, T, Hl, Wl = bs.latent_shape
    for t in range(T):
        for hg in range(Hl // 2):
            for wg in range(Wl // 2):
                cell = [lat[c, t, 2 * hg + dy, 2 * wg + dx] for c in range(C) for dy in range(2) for dx in range(2)]
                xrow = _loop_linear([cell], gw["w_patch"], gw["b_patch"])
                v = O.head(np.array(xrow), gw, t_head)[0]
                f = 0
                for c in range(C):
                    for dy in range(2):
                        for dx in range(2):
                            want = lat[c, t, 2 * hg + dy, 2 * wg + dx] - 0.5 * v[f]
                            assert abs(out[c, t, 2 * hg + dy, 2 * wg + dx] - want) < 1e-12
                            f += 1


# ------------------------------------------------------------- step / schedule

def _tiny_model(seed=0):
    bs = synth.BlockShape("tiny", D=32, H=2, dh=16, F=48, Lt=4, text_dim=24, grid=(2, 2, 3), C=2)
    blocks = [synth.stress_block_weights(bs, seed, b) for b in range(2)]
    gw = synth.glue_weights(bs, seed, std=0.2)
    text = synth.normal(seed, "text_raw", (bs.Lt, bs.text_dim))
    ctx = O.text_project(text, gw)
    t_mods = [synth.normal(seed, f"tm{i}", (6, bs.D), 0.05) for i in range(4)]
    t_heads = [synth.normal(seed, f"th{i}", (2, bs.D), 0.05) for i in range(4)]
    return bs, blocks, gw, ctx, t_mods, t_heads


def test_step_mask_ends():
    """All-compute masks give the unmasked step; the step only changes M_see tokens before
    the blend, and only M_edit tokens after it (Sec. 3.3.2)."""
    bs, blocks, gw, ctx, t_mods, t_heads = _tiny_model()
    lat = synth.latent(bs, 0)
    SL = synth.latent(bs, 0, "SL")
    ones = np.ones(bs.L, np.uint8)
    full = O.denoise_step(lat, blocks, gw, bs, ctx, t_mods[0], t_heads[0], -0.25)
    masked = O.denoise_step(lat, blocks, gw, bs, ctx, t_mods[0], t_heads[0], -0.25, mask_see=ones, mask_edit=ones, SL=SL)
    np.testing.assert_array_equal(full, masked)
    assert np.abs(full - lat).max() > 1e-3
    see = synth.exact_count_mask(bs.L, 7, seed=1)
    edit = see.copy()
    edit[O.region_compact(see)[:3]] = 0      # M_edit strictly inside M_see
    out = O.denoise_step(lat, blocks, gw, bs, ctx, t_mods[0], t_heads[0], -0.25, mask_see=see, mask_edit=edit, SL=SL)
    Me = O.expand_token_mask(edit, bs.grid, bs.patch, bs.C).astype(bool)
    np.testing.assert_array_equal(out[~Me], SL.astype(np.float64)[~Me])
    assert (out[Me] != SL.astype(np.float64)[Me]).all()
    # all-reuse edit mask returns the cached latent bit for bit
    out0 = O.denoise_step(lat, blocks, gw, bs, ctx, t_mods[0], t_heads[0], -0.25, mask_see=see,
                          mask_edit=np.zeros(bs.L, np.uint8), SL=SL)
    np.testing.assert_array_equal(out0, SL.astype(np.float64))


def test_schedule_run_stage1_and_miss():
    bs, blocks, gw, ctx, t_mods, t_heads = _tiny_model()
    lat = synth.latent(bs, 0)
    SL = synth.latent(bs, 0, "SL")
    sig = [1.0, 0.75, 0.5, 0.25, 0.0]
    # stage-1-only prefix: after K1 reused steps the latent is the source latent
    plan = [(1, 1.0, 1.0)]
    np.testing.assert_array_equal(O.run_schedule(plan, sig, lat, SL, blocks, gw, bs, ctx, t_mods, t_heads), SL)
    # a miss plan equals N plain steps
    _, _, plan = O.denoise_schedule(0.1, 0.75, 2)
    a = O.run_schedule(plan, sig, lat, SL, blocks, gw, bs, ctx, t_mods, t_heads)
    b = lat
    for i in range(2):
        b = O.denoise_step(b, blocks, gw, bs, ctx, t_mods[i], t_heads[i], sig[i + 1] - sig[i])
    np.testing.assert_array_equal(a, b)


# ------------------------------------------------------------------ region masks (Eq. 5, max-pool projection)

def _brute_dilate(m, r):
    T, H, W = m.shape
    out = np.zeros_like(m)
    for t in range(T):
        for y in range(H):
            for x in range(W):
                hit = 0
                for tt in range(max(0, t - r[0]), min(T, t + r[0] + 1)):
                    for yy in range(max(0, y - r[1]), min(H, y + r[1] + 1)):
                        for xx in range(max(0, x - r[2]), min(W, x + r[2] + 1)):
                            hit |= int(m[tt, yy, xx] != 0)
                out[t, y, x] = hit
    return out


def test_dilate_brute_force_and_scipy():
    from scipy import ndimage
    m = (synth.stream(0, "pin.dil").random((4, 9, 11)) < 0.08).astype(np.uint8)
    for r in [(0, 0, 0), (0, 1, 1), (1, 2, 3), (2, 0, 1), (0, 3, 0), (5, 12, 12)]:
        got = O.mask_dilate(m, r)
        np.testing.assert_array_equal(got, _brute_dilate(m, r))
        lib = ndimage.binary_dilation(m, structure=np.ones((2 * r[0] + 1, 2 * r[1] + 1, 2 * r[2] + 1), bool))
        np.testing.assert_array_equal(got, lib.astype(np.uint8))
    np.testing.assert_array_equal(O.mask_dilate(m, (0, 0, 0)), m)                 # K_0 = [1]: identity


def test_dilate_closed_forms():
    # one site -> the (2r+1) box around it, cut at the border; asymmetric radii hit the right axes
    m = np.zeros((5, 8, 10), np.uint8)
    m[2, 3, 4] = 1
    d = O.mask_dilate(m, (1, 2, 3))
    exp = np.zeros_like(m)
    exp[1:4, 1:6, 1:8] = 1
    np.testing.assert_array_equal(d, exp)
    assert d.sum() == 3 * 5 * 7
    m[:] = 0
    m[0, 0, 9] = 1                                                                  # corner: zero padding outside
    d = O.mask_dilate(m, (1, 1, 2))
    assert d.sum() == 2 * 2 * 3 and d[0:2, 0:2, 7:10].all()
    # box kernels compose: dilation by r1 then r2 is dilation by r1 + r2
    mm = synth.sparse_site_mask((4, 12, 12), 5, seed=3)
    np.testing.assert_array_equal(O.mask_dilate(O.mask_dilate(mm, (1, 1, 2)), (0, 2, 1)), O.mask_dilate(mm, (1, 3, 3)))
    # empty stays empty, full stays full
    assert O.mask_dilate(np.zeros((2, 3, 4), np.uint8), (1, 1, 1)).sum() == 0
    assert O.mask_dilate(np.ones((2, 3, 4), np.uint8), (1, 1, 1)).all()
    # any non-zero byte counts as set, the output is 0/1
    m3 = np.zeros((1, 3, 3), np.uint8)
    m3[0, 1, 1] = 200
    assert set(np.unique(O.mask_dilate(m3, (0, 1, 1)))) == {1}


def test_mask_hierarchy_containment():
    base = synth.pixel_key_masks(3, 24, 40, seed=1, n_obj=2)
    edit, see = O.mask_hierarchy(base, (0, 1, 1), (1, 3, 3))
    assert ((base != 0) <= (edit != 0)).all() and (edit <= see).all()              # M_see >= M_edit >= M_base
    assert edit.sum() > (base != 0).sum() and see.sum() > edit.sum()
    with pytest.raises(AssertionError):
        O.mask_hierarchy(base, (0, 2, 2), (0, 1, 3))                                # r' must dominate r


def test_maxpool_vs_torch_and_brute_force():
    m = (synth.stream(0, "pin.pool").random((9, 20, 28)) < 0.03).astype(np.uint8)
    # divisible and ragged windows against torch's max_pool3d (ceil_mode cuts windows at the edge)
    for win in [(1, 2, 2), (4, 8, 8), (2, 3, 5), (9, 20, 28), (1, 1, 1), (4, 16, 16)]:
        got = O.mask_maxpool(m, win)
        lib = TF.max_pool3d(torch.from_numpy(m)[None, None].float(), win, stride=win, ceil_mode=True)[0, 0]
        np.testing.assert_array_equal(got, lib.numpy().astype(np.uint8))
    # leading frame on its own (causal video VAE: 1 + 4k frames -> 1 + k latent frames)
    got = O.mask_maxpool(m, (4, 8, 8), t_lead=1)
    assert got.shape == (3, 3, 4)
    for t, (t0, t1) in enumerate([(0, 1), (1, 5), (5, 9)]):
        for y in range(3):
            for x in range(4):
                assert got[t, y, x] == int(m[t0:t1, 8 * y:8 * y + 8, 8 * x:8 * x + 8].any())
    assert O.pooled_extent(81, 4, 1) == 21 and O.pooled_extent(480, 16) == 30 and O.pooled_extent(17, 4) == 5
    # pooling keeps "any": set sites never vanish, empty windows stay empty
    assert got.any() == m.any()
    assert O.mask_maxpool(np.zeros((5, 8, 8), np.uint8), (4, 8, 8), 1).sum() == 0
    # two-step projection pixel -> latent -> token equals one pool with the product window
    a = O.mask_maxpool(O.mask_maxpool(m, (4, 8, 8), 1), (1, 2, 2))
    b = O.mask_maxpool(m, (4, 16, 16), 1)
    np.testing.assert_array_equal(a, b)


def test_keyframe_propagation():
    km = synth.pixel_key_masks(3, 12, 16, seed=2)
    fk = synth.frame_key_groups(9, 3)
    np.testing.assert_array_equal(fk, [0, 0, 0, 1, 1, 1, 2, 2, 2])
    fr = O.mask_propagate_keyframes(km, fk)
    assert fr.shape == (9, 12, 16)
    for f in range(9):
        np.testing.assert_array_equal(fr[f], (km[fk[f]] != 0).astype(np.uint8))
    with pytest.raises(AssertionError):
        O.mask_propagate_keyframes(km, np.array([0, 3]))


# ------------------------------------------------------------------ cache update (Sec. 3.1 "Cache Update")

def test_cache_insert_then_lookup():
    cache = np.zeros((6, 32), np.float32)                     # a zero-filled cache is an empty one
    lats = np.zeros((6, 2, 3), np.float32)
    q = synth.normal(0, "ins.q", (32,))
    j0, m0, hit0 = O.cache_lookup(cache, q, 0.75)
    assert not hit0 and m0 == -np.inf
    lat = synth.normal(0, "ins.lat", (2, 3))
    c2, l2 = O.cache_insert(cache, lats, 4, q, lat)
    assert not cache.any() and not lats.any()                 # inputs untouched
    j, m, hit = O.cache_lookup(c2, q, 0.75)
    assert (j, hit) == (4, True) and abs(m - 1.0) < 1e-6      # the stored prompt is found with cosine 1
    np.testing.assert_array_equal(l2[4], lat)
    np.testing.assert_array_equal(np.delete(c2, 4, 0), np.delete(cache, 4, 0))   # every other entry unchanged
    np.testing.assert_array_equal(np.delete(l2, 4, 0), np.delete(lats, 4, 0))
    # replacing an entry: the old prompt no longer matches
    q2 = synth.normal(1, "ins.q", (32,))
    c3, _ = O.cache_insert(c2, l2, 4, q2, lat)
    assert not O.cache_lookup(c3, q, 0.75)[2] and O.cache_lookup(c3, q2, 0.75)[0] == 4
    with pytest.raises(AssertionError):
        O.cache_insert(cache, lats, 6, q, lat)


def test_run_schedule_snapshot_is_the_prefix_run():
    # the latent kept by a cache update after k steps equals running only the first k steps
    bs = synth.SHAPES["c1"]
    blocks = [synth.block_weights(bs, 0, 0)]
    gw = synth.glue_weights(bs, 0)
    ctx = synth.round_bf16(synth.normal(0, "snap.ctx", (bs.Lt, bs.D), 1.0))
    t_mods = synth.normal(0, "t_mods", (4, 6, bs.D), 0.02)
    t_heads = synth.normal(0, "t_heads", (4, 2, bs.D), 0.02)
    sig = [1.0, 0.75, 0.5, 0.25, 0.0]
    lat0 = synth.latent(bs, 0, "noise", std=1.0)
    plan = [(3, 1.0, 1.0)] * 4
    full, snap = O.run_schedule(plan, sig, lat0, None, blocks, gw, bs, ctx, t_mods, t_heads, store_after=2)
    two = O.run_schedule(plan[:2], sig[:3], lat0, None, blocks, gw, bs, ctx, t_mods[:2], t_heads[:2])
    np.testing.assert_array_equal(snap, two)
    assert not np.array_equal(full, snap)
    _, last = O.run_schedule(plan, sig, lat0, None, blocks, gw, bs, ctx, t_mods, t_heads, store_after=4)
    np.testing.assert_array_equal(last, full)


# ------------------------------------------------------------------ sampler: DPM-Solver++ on the rectified-flow path (Sec. 4.1)

def _gauss_x0(x, sig, mu, s):
    """E[x0 | x_sigma] for data ~ N(mu, s^2) on the path x = (1 - sigma) x0 + sigma eps."""
    a = 1.0 - sig
    return mu + a * s * s / (a * a * s * s + sig * sig) * (x - a * mu)


def _gauss_flow_exact(x_a, sig_a, sig_b, mu, s):
    """The probability-flow ODE keeps (x - alpha mu) / std(x_sigma) fixed for Gaussian data."""
    f = lambda sg: math.sqrt((1.0 - sg) ** 2 * s * s + sg * sg)
    return (1.0 - sig_b) * mu + f(sig_b) * (x_a - (1.0 - sig_a) * mu) / f(sig_a)


def _solve_gauss(n, order, grid="sigma"):
    mu, s = 0.7, 0.5
    if grid == "sigma":
        sig = np.linspace(0.9, 0.1, n + 1)          # uniform in sigma: h changes from step to step, r != 1
    else:
        u = np.linspace(0.0, 1.0, n + 1) ** 1.5
        sig = 0.9 - 0.8 * u
    x = np.array([1.3, -0.4, 0.05])
    start, prev = x.copy(), None
    for i in range(n):
        x0 = _gauss_x0(x, sig[i], mu, s)
        if order == 2 and prev is not None:
            x = O.dpmpp_2m(x, x0, prev, sig[i - 1], sig[i], sig[i + 1])
        else:
            x = O.dpmpp_first_order(x, x0, sig[i], sig[i + 1])
        prev = x0
    return np.abs(x - _gauss_flow_exact(start, 0.9, 0.1, mu, s)).max()


@pytest.mark.parametrize("grid", ["sigma", "warped"])
def test_dpmpp_convergence_order_on_gaussian_flow(grid):
    """Against the closed-form flow of Gaussian data: halving the step halves the error of the
    first-order update and quarters that of the multistep one. A wrong sign or a wrong r in the
    extrapolation term leaves only first-order convergence."""
    e1 = [_solve_gauss(n, 1, grid) for n in (64, 128, 256)]
    e2 = [_solve_gauss(n, 2, grid) for n in (64, 128, 256)]
    for a, b in zip(e1, e1[1:]):
        assert 1.8 < a / b < 2.2
    for a, b in zip(e2, e2[1:]):
        assert 3.6 < a / b < 4.4
    assert e2[-1] < 0.02 * e1[-1]


def test_dpmpp_closed_forms():
    rng = synth.stream(3, "dpmpp")
    x0 = rng.standard_normal(11)
    eps = rng.standard_normal(11)
    # constant data prediction: every order lands on the path through (x0, eps) exactly
    sig = [1.0, 0.83, 0.6, 0.41, 0.2, 0.0]
    x = sig[0] * eps + (1 - sig[0]) * x0
    for i in range(5):
        if i == 0 or sig[i + 1] == 0.0:
            x = O.dpmpp_first_order(x, x0, sig[i], sig[i + 1])
        else:
            x = O.dpmpp_2m(x, x0, x0, sig[i - 1], sig[i], sig[i + 1])
        np.testing.assert_allclose(x, sig[i + 1] * eps + (1 - sig[i + 1]) * x0, rtol=0, atol=1e-14)
    # first order on the rectified-flow path is the Euler step in the velocity
    xs = rng.standard_normal(11)
    v = rng.standard_normal(11)
    for s_, t_ in ((1.0, 0.7), (0.7, 0.3), (0.3, 0.0), (1.0, 0.0)):
        got = O.dpmpp_first_order(xs, O.velocity_to_x0(xs, v, s_), s_, t_)
        np.testing.assert_allclose(got, xs + (t_ - s_) * v, rtol=0, atol=1e-14)
    # a step that ends at sigma = 0 returns the data prediction itself
    np.testing.assert_allclose(O.dpmpp_first_order(xs, x0, 0.4, 0.0), x0, rtol=0, atol=1e-15)
    # equal predictions: nothing to extrapolate; history taken at sigma = 1 (lambda = -inf) has no weight
    a = O.dpmpp_2m(xs, x0, x0, 0.9, 0.6, 0.3)
    np.testing.assert_allclose(a, O.dpmpp_first_order(xs, x0, 0.6, 0.3), rtol=0, atol=1e-14)
    b = O.dpmpp_2m(xs, x0, eps, 1.0, 0.6, 0.3)
    np.testing.assert_allclose(b, O.dpmpp_first_order(xs, x0, 0.6, 0.3), rtol=0, atol=1e-14)
    # equal steps in lambda (r = 1): D = 1.5 x0 - 0.5 x0_prev
    lam = np.array([-1.0, -0.2, 0.6])
    sg = 1.0 / (1.0 + np.exp(lam))                 # lambda = log((1 - sigma) / sigma)
    np.testing.assert_allclose(O.flow_lambda(sg), lam, atol=1e-14)
    c = O.dpmpp_2m(xs, x0, eps, sg[0], sg[1], sg[2])
    np.testing.assert_allclose(c, O.dpmpp_update(xs, 1.5 * x0 - 0.5 * eps, sg[1], sg[2]), rtol=0, atol=1e-13)
    # the velocity of the path is eps - x0
    xt = 0.35 * eps + 0.65 * x0
    np.testing.assert_allclose(O.velocity_to_x0(xt, eps - x0, 0.35), x0, atol=1e-14)


def test_cfg_combine_ends():
    rng = synth.stream(4, "cfg")
    vc, vu = rng.standard_normal(9), rng.standard_normal(9)
    np.testing.assert_array_equal(O.cfg_combine(vc, vu, 0.0), vu)
    np.testing.assert_allclose(O.cfg_combine(vc, vu, 1.0), vc, atol=1e-15)
    np.testing.assert_allclose(O.cfg_combine(vc, vu, 5.0) - vc, 4.0 * (vc - vu), atol=1e-14)
    np.testing.assert_array_equal(O.cfg_combine(vc, vc, 7.5), vc)


def test_step_dpmpp_reduces_to_the_euler_step_and_tracks_history():
    bs, blocks, gw, ctx, t_mods, t_heads = _tiny_model()
    lat = synth.latent(bs, 0)
    SL = synth.latent(bs, 0, "SL")
    junk = synth.latent(bs, 0, "x0prev")
    none = np.zeros(bs.L, np.uint8)
    ones = np.ones(bs.L, np.uint8)
    euler = O.denoise_step(lat, blocks, gw, bs, ctx, t_mods[0], t_heads[0], 0.5 - 0.75)
    for order, hist in ((1, ones), (2, none)):          # first order asked for, or no history to use
        out, x0h, h = O.denoise_step_dpmpp(lat, blocks, gw, bs, ctx, t_mods[0], t_heads[0], 1.0, 0.75, 0.5, junk, hist,
                                           order=order)
        np.testing.assert_allclose(out, euler, rtol=0, atol=1e-12)
        assert h.all()
        v = O.model_velocity(lat, np.arange(bs.L), blocks, gw, bs, ctx, t_mods[0], t_heads[0])
        np.testing.assert_allclose(x0h, lat - 0.75 * O.unpatchify(v, lat.shape, bs.patch), rtol=0, atol=1e-12)
    # with history the second-order term moves the result, and only on tokens that have it
    part = synth.exact_count_mask(bs.L, 5, seed=2)
    out2, _, _ = O.denoise_step_dpmpp(lat, blocks, gw, bs, ctx, t_mods[0], t_heads[0], 1.0 - 1e-3, 0.75, 0.5, junk, part)
    tok_changed = np.abs(O.patchify(out2 - euler, bs.patch)).max(axis=1) > 1e-9
    np.testing.assert_array_equal(tok_changed, part != 0)
    # the last step (sigma -> 0) is first order whatever the history
    last, _, _ = O.denoise_step_dpmpp(lat, blocks, gw, bs, ctx, t_mods[0], t_heads[0], 0.5, 0.25, 0.0, junk, ones)
    np.testing.assert_allclose(last, O.denoise_step(lat, blocks, gw, bs, ctx, t_mods[0], t_heads[0], -0.25), atol=1e-12)
    # stage 2: computed tokens get history, the others lose it; outside M_edit the latent is the source latent
    see = synth.exact_count_mask(bs.L, 7, seed=1)
    edit = see.copy()
    edit[O.region_compact(see)[:3]] = 0
    out3, x0h3, h3 = O.denoise_step_dpmpp(lat, blocks, gw, bs, ctx, t_mods[0], t_heads[0], 1.0, 0.75, 0.5, junk, ones,
                                          mask_see=see, mask_edit=edit, SL=SL)
    np.testing.assert_array_equal(h3, see)
    Me = O.expand_token_mask(edit, bs.grid, bs.patch, bs.C).astype(bool)
    Ms = O.expand_token_mask(see, bs.grid, bs.patch, bs.C).astype(bool)
    np.testing.assert_array_equal(out3[~Me], SL.astype(np.float64)[~Me])
    np.testing.assert_array_equal(x0h3[~Ms], junk.astype(np.float64)[~Ms])
    assert (x0h3[Ms] != junk.astype(np.float64)[Ms]).all()
    # guidance 1 with any unconditional prompt is the conditional step; equal prompts cancel the guidance scale
    ctx_u = O.text_project(synth.normal(5, "text_uncond", (bs.Lt, bs.text_dim)), gw)
    g1, _, _ = O.denoise_step_dpmpp(lat, blocks, gw, bs, ctx, t_mods[0], t_heads[0], 1.0, 0.75, 0.5, junk, none,
                                    text_ctx_uncond=ctx_u, guidance=1.0)
    np.testing.assert_allclose(g1, euler, rtol=0, atol=1e-12)
    g5, _, _ = O.denoise_step_dpmpp(lat, blocks, gw, bs, ctx, t_mods[0], t_heads[0], 1.0, 0.75, 0.5, junk, none,
                                    text_ctx_uncond=ctx, guidance=5.0)
    np.testing.assert_allclose(g5, euler, rtol=0, atol=1e-12)
    g3, _, _ = O.denoise_step_dpmpp(lat, blocks, gw, bs, ctx, t_mods[0], t_heads[0], 1.0, 0.75, 0.5, junk, none,
                                    text_ctx_uncond=ctx_u, guidance=3.0)
    gu, _, _ = O.denoise_step_dpmpp(lat, blocks, gw, bs, ctx_u, t_mods[0], t_heads[0], 1.0, 0.75, 0.5, junk, none)
    np.testing.assert_allclose(g3, gu + 3.0 * (euler - gu), rtol=0, atol=1e-11)    # the update is linear in v


def test_run_schedule_dpmpp_first_order_is_the_euler_run():
    bs, blocks, gw, ctx, t_mods, t_heads = _tiny_model()
    lat = synth.latent(bs, 0)
    SL = synth.latent(bs, 0, "SL")
    sig = [1.0, 0.8, 0.55, 0.3, 0.0]
    see = synth.exact_count_mask(bs.L, 7, seed=1)
    edit = see.copy()
    edit[O.region_compact(see)[:2]] = 0
    plan = [(1, 1.0, 1.0), (2, 1.2, 1.1), (3, 1.1, 1.0), (3, 1.0, 1.0)]
    ks = lambda g: synth.tdiff_scale(bs.Lt, g, seed=0)
    a = O.run_schedule(plan, sig, lat, SL, blocks, gw, bs, ctx, t_mods, t_heads, mask_see=see, mask_edit=edit,
                       key_scale_of=ks)
    b = O.run_schedule_dpmpp(plan, sig, lat, SL, blocks, gw, bs, ctx, t_mods, t_heads, order=1, mask_see=see,
                             mask_edit=edit, key_scale_of=ks)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-11)
    c = O.run_schedule_dpmpp(plan, sig, lat, SL, blocks, gw, bs, ctx, t_mods, t_heads, order=2, mask_see=see,
                             mask_edit=edit, key_scale_of=ks)
    assert np.abs(c - a).max() > 1e-6          # step 2 (stage 3, after a stage-2 step) extrapolates on the M_see tokens


# ------------------------------------------------------------------ several stored depths per entry (Sec. 3.1 "Cache Update")

@pytest.mark.parametrize("N", [4, 8, 50])
def test_schedule_with_stored_depths(N):
    tau = 0.75
    every = list(range(1, N + 1))
    prev = -1
    for m in np.linspace(0.0, 1.0, 41):
        K1, K2, plan = O.denoise_schedule(m, tau, N)
        # every depth stored: nothing changes
        assert O.denoise_schedule(m, tau, N, stored_steps=every) == (K1, K2, plan)
        for stored in ([1], [2], [1, 3], [N // 2, N // 4 + 1], [N]):
            k1, k2, pl = O.denoise_schedule(m, tau, N, stored_steps=stored)
            assert k1 in stored or (k1, k2) == (0, 0)
            assert k1 <= K1 and 0 <= k1 <= k2 <= max(N - 1, 0)
            ok = [k for k in stored if 1 <= k <= K1]
            assert k1 == (max(ok) if ok else 0)
            if ok:
                assert k2 - k1 >= K2 - K1                       # the region stage is never shortened
                if K2 < N - 1:
                    assert k2 - k1 == K2 - K1                   # and keeps its length where Eq. 1 was not clipped
                assert [p[0] for p in pl] == [1] * k1 + [2] * (k2 - k1) + [3] * (N - k2)
                # the factors are those of a schedule whose Eq. 1 lands on k1 directly
                for i in range(k1, N):
                    w = max(0.0, 1.0 - (i - k1) / max(1, k2 - k1))
                    assert pl[i][1] >= 1.0 and (w > 0 or pl[i][1] == 1.0)
            else:
                assert pl == [(3, 1.0, 1.0)] * N
        k1, _, _ = O.denoise_schedule(m, tau, N, stored_steps=[1, 3])
        assert k1 >= prev                      # still monotone in the similarity
        prev = k1
    assert O.denoise_schedule(0.5, tau, N, stored_steps=every)[:2] == (0, 0)      # a miss stays a miss


def test_run_schedule_snapshots_at_several_depths():
    bs, blocks, gw, ctx, t_mods, t_heads = _tiny_model()
    lat = synth.latent(bs, 0)
    sig = [1.0, 0.75, 0.5, 0.25, 0.0]
    plan = [(3, 1.0, 1.0)] * 4
    final, snaps = O.run_schedule(plan, sig, lat, None, blocks, gw, bs, ctx, t_mods, t_heads, store_after=[1, 3])
    one, s1 = O.run_schedule(plan, sig, lat, None, blocks, gw, bs, ctx, t_mods, t_heads, store_after=1)
    _, s3 = O.run_schedule(plan, sig, lat, None, blocks, gw, bs, ctx, t_mods, t_heads, store_after=3)
    np.testing.assert_array_equal(final, one)
    np.testing.assert_array_equal(snaps[0], s1)
    np.testing.assert_array_equal(snaps[1], s3)
    # resuming from the depth-3 state reproduces the rest of the run
    rest = O.denoise_step(snaps[1], blocks, gw, bs, ctx, t_mods[3], t_heads[3], sig[4] - sig[3])
    np.testing.assert_array_equal(rest, final)


# ------------------------------------------------------------------ batched top-k retrieval

def test_lookup_topk_brute_force_and_reductions():
    rng = synth.stream(21, "topk")
    cache = rng.standard_normal((37, 12))
    cache[9] = cache[4]                      # equal rows: equal scores, lower index first
    cache[20] = 2.0 * cache[4]               # cosine ignores the scale (a power of two keeps the tie exact)
    cache[30] = 0.0                          # zero norm: -inf, sorted last
    queries = np.vstack([rng.standard_normal((5, 12)), cache[4][None], np.zeros((1, 12))])
    k = 6
    idx, sc, hit = O.cache_lookup_topk(cache, queries, 0.6, k)
    assert idx.shape == (7, k) and sc.shape == (7, k) and hit.shape == (7,)
    for qi, q in enumerate(queries):
        # brute force: plain Python cosine, selection by repeated scan
        scores = [_brute_lookup(cache[j:j + 1], q)[1] for j in range(cache.shape[0])]
        left = list(range(cache.shape[0]))
        for r in range(k):
            best = left[0]
            for j in left:
                if scores[j] > scores[best]:
                    best = j
            left.remove(best)
            assert idx[qi, r] == best and (sc[qi, r] == scores[best] or abs(sc[qi, r] - scores[best]) < 1e-12)
        # column 0 is the single-query lookup
        j, m, h = O.cache_lookup(cache, q, 0.6)
        assert (idx[qi, 0], hit[qi]) == (j, h) and sc[qi, 0] == m
        assert all(sc[qi, r] >= sc[qi, r + 1] for r in range(k - 1))
    assert list(idx[5, :3]) == [4, 9, 20] and np.allclose(sc[5, :3], 1.0) and hit[5]
    assert np.isinf(sc[6]).all() and list(idx[6]) == [0, 1, 2, 3, 4, 5] and not hit[6]   # zero query: all -inf, by index
    # k beyond the cache size pads with (-1, -inf); k = 1 and an empty cache
    idx, sc, hit = O.cache_lookup_topk(cache[:3], queries[:2], 0.6, 5)
    assert (idx[:, 3:] == -1).all() and np.isinf(sc[:, 3:]).all() and sorted(idx[0, :3]) == [0, 1, 2]
    idx, sc, hit = O.cache_lookup_topk(cache[:0], queries[:2], 0.6, 2)
    assert (idx == -1).all() and np.isinf(sc).all() and not hit.any()
    # a batch is the per-query results stacked
    a = O.cache_lookup_topk(cache, queries, 0.6, 3)
    for qi in range(queries.shape[0]):
        b = O.cache_lookup_topk(cache, queries[qi:qi + 1], 0.6, 3)
        assert (a[0][qi] == b[0][0]).all() and (a[1][qi] == b[1][0]).all() and a[2][qi] == b[2][0]


# ------------------------------------------------------------------ timestep modulation

def test_time_mod_vs_torch_and_closed_forms():
    bs = synth.BlockShape("tiny", D=32, H=2, dh=16, F=48, Lt=4, text_dim=24, grid=(2, 2, 3), C=2)
    tw = synth.time_weights(bs, 0, freq_dim=16, std=0.3)
    f0 = O.sinusoidal_features(0.0, 16)
    np.testing.assert_array_equal(f0, np.concatenate([np.ones(8), np.zeros(8)]))        # cos 0 = 1, sin 0 = 0
    f = O.sinusoidal_features(37.5, 16)
    for i in range(8):                                                                    # written out with math.*
        w = 10000.0 ** (-i / 8)
        assert abs(f[i] - math.cos(37.5 * w)) < 1e-12 and abs(f[8 + i] - math.sin(37.5 * w)) < 1e-12
    np.testing.assert_allclose(f[:8] ** 2 + f[8:] ** 2, 1.0, atol=1e-12)
    assert f[0] == math.cos(37.5) and abs(f[7] - math.cos(37.5 * 10000.0 ** (-7 / 8))) < 1e-12
    np.testing.assert_allclose(O.silu(np.array([-2.0, 0.0, 3.0])), TF.silu(torch.tensor([-2.0, 0.0, 3.0], dtype=torch.float64)).numpy(),
                               atol=1e-15)
    t_mod, t_head = O.time_mod(421.0, tw, bs.D, 16)
    T = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    ft = torch.cat([torch.cos(421.0 * T(10000.0 ** (-np.arange(8) / 8))), torch.sin(421.0 * T(10000.0 ** (-np.arange(8) / 8)))])
    e = TF.linear(TF.silu(TF.linear(ft, T(tw["w_t1"]), T(tw["b_t1"]))), T(tw["w_t2"]), T(tw["b_t2"]))
    tm = TF.linear(TF.silu(e), T(tw["w_tp"]), T(tw["b_tp"])).reshape(6, bs.D)
    np.testing.assert_allclose(t_mod, tm.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(t_head, torch.stack([e, e]).numpy(), rtol=0, atol=1e-12)
    assert t_mod.shape == (6, bs.D) and t_head.shape == (2, bs.D)
    # row r of t_mod comes from rows [r D, (r + 1) D) of the projection
    np.testing.assert_allclose(t_mod[4], O.linear(O.silu(t_head[0]), tw["w_tp"][4 * bs.D:5 * bs.D], tw["b_tp"][4 * bs.D:5 * bs.D]),
                               atol=1e-12)
    # different timesteps give different modulation
    assert np.abs(O.time_mod(420.0, tw, bs.D, 16)[0] - t_mod).max() > 1e-4


# ---------------------------------------------- low-precision embedding storage with exact re-rank

def _nearest_even_brute(x, values):
    """Nearest of the sorted representable `values` to x, ties to the one whose position is even."""
    best, bi = None, None
    for i, v in enumerate(values):
        d = abs(v - x)
        if best is None or d < best or (d == best and i % 2 == 0 and bi % 2 == 1):
            best, bi = d, i
    return bi


def test_fp8_e4m3_format_and_rounding():
    """The FP8 E4M3 table against the format's published corner values, the encoder against a brute-force nearest
    search and against torch's conversion; decode(encode(v)) = v on every representable value."""
    mags = O.fp8_e4m3_decode(np.arange(127, dtype=np.uint8))
    assert mags[0] == 0.0 and mags[1] == 2.0 ** -9 and mags[7] == 7 * 2.0 ** -9          # subnormals
    assert mags[8] == 2.0 ** -6 and mags[0x38] == 1.0 and mags[0x7E] == 448.0            # smallest normal, one, largest
    assert (np.diff(mags) > 0).all()
    np.testing.assert_array_equal(O.fp8_e4m3_decode(np.arange(128, 255, dtype=np.uint8)), -mags)
    np.testing.assert_array_equal(O.fp8_e4m3_encode(mags), np.arange(127, dtype=np.uint8))
    np.testing.assert_array_equal(O.fp8_e4m3_encode(-mags[1:]), np.arange(129, 255, dtype=np.uint8))
    rng = synth.stream(31, "fp8")
    xs = np.concatenate([rng.normal(size=300) * 10.0 ** rng.uniform(-4, 2.6, size=300),
                         (mags[:-1] + mags[1:]) / 2, [448.0, 460.0, 1e9, 2.0 ** -10, 2.0 ** -11, 0.0]])
    enc = O.fp8_e4m3_encode(xs)
    for x, e in zip(xs, enc):
        want = _nearest_even_brute(min(abs(x), 448.0), list(mags))
        assert (e & 0x7F) == want and bool(e & 0x80) == bool(np.signbit(x)), (x, e, want)
    if hasattr(torch, "float8_e4m3fn"):
        y = np.clip(xs, -448, 448).astype(np.float32)
        t8 = torch.from_numpy(y).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        np.testing.assert_array_equal(O.fp8_e4m3_encode(y), t8)


def test_bf16_rounding_vs_brute_force_and_torch():
    rng = synth.stream(32, "bf16")
    x = (rng.normal(size=2000) * 10.0 ** rng.uniform(-6, 6, size=2000)).astype(np.float32)
    enc = O.bf16_encode(x)
    np.testing.assert_array_equal(enc, torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))
    # brute force on a few: the two neighbouring bf16 values around x, nearest wins, ties to the even code
    for v, e in list(zip(x, enc))[:200]:
        trunc = int(np.float32(v).view(np.uint32)) >> 16
        lo, hi = O.bf16_decode(np.uint16(trunc)), O.bf16_decode(np.uint16(trunc + 1))
        dl, dh = abs(float(v) - lo), abs(hi - float(v))
        want = trunc if dl < dh or (dl == dh and trunc % 2 == 0) else trunc + 1
        assert e == want
    exact_tie = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8], np.float32)          # halfway cases
    np.testing.assert_array_equal(O.bf16_decode(O.bf16_encode(exact_tie)), [1.0, 1.0 + 2.0 ** -6])


def _same_lookup(a, b):
    """Index and hit exactly; the score up to the rounding order of the matrix product (a dot product taken inside a
    product over a few rows and inside one over all rows may differ in the last bit)."""
    return a[0] == b[0] and a[2] == b[2] and (a[1] == b[1] or abs(a[1] - b[1]) <= 1e-14)


@pytest.mark.parametrize("fmt", O.LOWPREC_FORMATS)
def test_lowprec_lookup_is_the_exact_lookup(fmt):
    """The two-stage retrieval returns cache_lookup's result on clustered caches, on near-duplicate rows that the
    low-precision copy cannot tell apart (or ranks the wrong way round), with duplicates, zero rows and a zero
    query; the score change stays inside the bound the margin is derived from."""
    for seed, (N, d) in enumerate([(64, 32), (300, 256), (257, 768)]):
        cache = synth.cache_embeddings(N, d, seed=seed)
        codes = O.cache_lowprec_encode(cache, fmt)
        assert codes.shape == cache.shape and codes.dtype == (np.uint16 if fmt == "bf16" else np.uint8)
        half = O.lowprec_margin(fmt, d) / 2
        for trial, near in enumerate((N // 2, None, 0, N - 1)):
            q = synth.cache_query(cache, seed=seed, near=near, trial=trial)
            exact = O.cosine_scores(cache, q)
            approx = O.cosine_scores(O.cache_lowprec_decode(codes, fmt), q)
            assert np.abs(approx - exact).max() <= half
            j, m, hit, n = O.cache_lookup_lowprec(cache, codes, fmt, q, 0.75)
            assert _same_lookup((j, m, hit), O.cache_lookup(cache, q, 0.75)) and 1 <= n <= N
    # adversarial: rows that differ from the query's source by less than the storage resolution
    cache = synth.cache_embeddings(40, 64, seed=9)
    q = cache[7].copy()
    for k, eps in enumerate((1e-4, 3e-4, 1e-3)):
        cache[20 + k] = cache[7] + eps * synth.normal(9, f"adv{k}", (64,))
    cache[33] = cache[7]                                   # an exact duplicate at a higher index
    codes = O.cache_lowprec_encode(cache, fmt)
    approx = O.cosine_scores(O.cache_lowprec_decode(codes, fmt), q)
    j, m, hit, n = O.cache_lookup_lowprec(cache, codes, fmt, q, 0.75)
    assert _same_lookup((j, m, hit), O.cache_lookup(cache, q, 0.75)) and (j, hit) == (7, True) and n >= 5
    assert O.cache_lookup_lowprec(cache, codes, fmt, q, 0.75, margin=0.0)[3] >= 1
    # the approximate ranking alone would not do: with these rows some other entry ties or beats row 7
    assert (approx[[20, 21, 22, 33]] >= approx[7] - 1e-12).any()
    # zero rows, zero query, empty cache
    cache[3] = 0
    codes = O.cache_lowprec_encode(cache, fmt)
    assert not codes[3].any()
    assert _same_lookup(O.cache_lookup_lowprec(cache, codes, fmt, q, 0.75)[:3], O.cache_lookup(cache, q, 0.75))
    assert O.cache_lookup_lowprec(cache, codes, fmt, np.zeros(64), 0.75)[:3] == O.cache_lookup(cache, np.zeros(64), 0.75)
    assert O.cache_lookup_lowprec(np.zeros((0, 64)), np.zeros((0, 64), np.uint8), fmt, q, 0.75) == (-1, -math.inf, False, 0)


def test_fp8_row_scaling():
    """Each row uses the whole FP8 range (its largest magnitude encodes as 448) whatever its norm, and rows that
    differ only by a positive factor encode alike up to the fp32 rounding of the scale."""
    cache = synth.cache_embeddings(16, 128, seed=4)
    codes = O.cache_lowprec_encode(cache, "fp8")
    assert ((codes & 0x7F).max(axis=1) == 0x7E).all()
    scaled = (cache * np.float32(1024.0)).astype(np.float32)          # a power of two: exactly the same codes
    np.testing.assert_array_equal(O.cache_lowprec_encode(scaled, "fp8"), codes)
