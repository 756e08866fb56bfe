"""Where the floating-point tolerances of the GPU parity tests come from, shown on the CPU alone.

The GPU path keeps the residual stream, the normalisations and the softmax in fp32 but feeds
bf16 operands to the matrix pipe. Here the ORACLE's own fp64 arithmetic is re-run with those
operands rounded to bf16 at exactly the points where the data flow of a block stores bf16 (the
modulated LayerNorm output, the projections, the normalised q / k, the probabilities that
enter P V, the attention output, the FFN hidden), and compared with the unrounded oracle. No
HIP code is involved: whatever error appears is what ANY implementation with bf16 operands
shows on these inputs, i.e. the floor under the tolerance a parity test can ask for.

Two facts are pinned:
* with the benchmark's random-init recipe the rounded run stays inside the benchmark spec's bounds
  (max-abs 2e-2, rel-L2 5e-3) with room to spare, so those bounds are meaningful there;
* with the "stress" recipe (q / k gains of 2, gates ~1, biases, key amplification 1.5) the
  rounded run itself exceeds max-abs 2e-2: the wider bound the stress parity test uses
  (max|ref| * 2^-6, rel-L2 1e-2) is set by the operand precision, not by a kernel defect.
CPU only."""
import math

import numpy as np
import pytest

import synth
from oracle import chorus_oracle as O

F64 = np.float64


def r16(a):
    """Round to bf16 (nearest even) and return as float64."""
    return synth.round_bf16(np.asarray(a, np.float32)).astype(F64)


def attention_bf16_operands(q, k, v, H, dh, key_scale=None):
    """softmax(g_j q k^T / sqrt(dh)) v with q, k, v given as bf16 values and the unnormalised probabilities rounded
    to bf16 before they multiply v, the row sum taken from the unrounded ones (what a flash-style kernel does)."""
    Lq, Lk = q.shape[0], k.shape[0]
    qh = q.reshape(Lq, H, dh).transpose(1, 0, 2)
    kh = k.reshape(Lk, H, dh).transpose(1, 0, 2)
    vh = v.reshape(Lk, H, dh).transpose(1, 0, 2)
    out = np.empty((H, Lq, dh), F64)
    for h in range(H):
        s = qh[h] @ kh[h].T / math.sqrt(dh)
        if key_scale is not None:
            s = s * np.asarray(key_scale, F64)[None, :]
        p = np.exp(s - s.max(-1, keepdims=True))
        out[h] = (r16(p) @ vh[h]) / p.sum(-1, keepdims=True)
    return out.transpose(1, 0, 2).reshape(Lq, H * dh)


def block_with_bf16_operands(x, w, bs, text_ctx, t_mod, token_idx=None, key_scale=None, gamma_o=1.0):
    """The oracle's block, step by step, with every tensor that the data flow of a block keeps in bf16 rounded to
    bf16; everything else (residual stream, norms, softmax statistics, accumulation) stays fp64."""
    D, H, dh, grid = bs.D, bs.H, bs.dh, bs.grid
    x = np.asarray(x, F64)
    Ls = x.shape[0]
    idx = np.arange(Ls) if token_idx is None else np.asarray(token_idx, np.int64)
    sh1, sc1, g1, sh2, sc2, g2 = np.asarray(w["mod_table"], F64) + np.asarray(t_mod, F64)
    h = r16(O.layernorm(x) * (1.0 + sc1) + sh1)
    qkv = r16(O.linear(h, w["w_qkv"], w["b_qkv"]))
    q = r16(O.rope3d(O.rmsnorm(qkv[:, :D], w["g_q"]), idx, grid, H, dh))
    k = r16(O.rope3d(O.rmsnorm(qkv[:, D:2 * D], w["g_k"]), idx, grid, H, dh))
    ao = r16(attention_bf16_operands(q, k, qkv[:, 2 * D:], H, dh))
    x = x + g1 * O.linear(ao, w["w_o"], w["b_o"])
    hc = r16(O.layernorm(x) * np.asarray(w["ln3_w"], F64) + np.asarray(w["ln3_b"], F64))
    qc = r16(O.rmsnorm(r16(O.linear(hc, w["w_cq"], w["b_cq"])), w["g_cq"]))
    tkv = r16(O.linear(r16(text_ctx), w["w_ckv"], w["b_ckv"]))
    kc = r16(O.rmsnorm(tkv[:, :D], w["g_ck"]))
    ao = r16(attention_bf16_operands(qc, kc, tkv[:, D:], H, dh, key_scale))
    x = x + gamma_o * O.linear(ao, w["w_co"], w["b_co"])
    h2 = r16(O.layernorm(x) * (1.0 + sc2) + sh2)
    f = r16(O.gelu_tanh(O.linear(h2, w["w_1"], w["b_1"])))
    return x + g2 * O.linear(f, w["w_2"], w["b_2"])


def _errs(got, ref):
    return float(np.abs(got - ref).max()), float(np.linalg.norm(got - ref) / np.linalg.norm(ref))


def test_rounding_points_do_not_change_the_exact_cases():
    """The rounded pipeline is the oracle's when nothing needs rounding: one token, one text token (both softmaxes
    are 1.0), inputs that are bf16 values -- then only the GEMM outputs are rounded and the result stays within
    bf16 precision of the oracle; and with all gates zero it is the input."""
    bs = synth.BlockShape("t", D=32, H=2, dh=16, F=64, Lt=1, text_dim=8, grid=(1, 1, 1))
    w = synth.stress_block_weights(bs, 1)
    inp = synth.block_inputs(bs, 1, x_std=1.0)
    ref = O.dit_block(inp["x"], w, bs, inp["text_ctx"], inp["t_mod"], gamma_o=1.5)
    got = block_with_bf16_operands(inp["x"], w, bs, inp["text_ctx"], inp["t_mod"], gamma_o=1.5)
    a, r = _errs(got, ref)
    assert r < 1e-2 and a < 5e-2
    w0 = dict(w)
    mt = w["mod_table"].copy()
    mt[2] = -inp["t_mod"][2]
    mt[5] = -inp["t_mod"][5]
    w0["mod_table"] = mt
    got = block_with_bf16_operands(inp["x"], w0, bs, inp["text_ctx"], inp["t_mod"], gamma_o=0.0)
    np.testing.assert_array_equal(got, np.asarray(inp["x"], F64))


@pytest.mark.parametrize("stress", [False, True])
def test_bf16_operand_floor_on_the_small_grid(stress):
    """1.3B widths on the 5 x 12 x 20 grid, TGAA 1.5 on 8 text tokens, gamma_o 1.5: the inputs of the GPU test
    test_block_1p3b_widths_small_grid."""
    bs = synth.SHAPES["wan1p3b_small"]
    w = synth.stress_block_weights(bs, 0) if stress else synth.block_weights(bs, 0)
    inp = synth.block_inputs(bs, 0)
    g = synth.tdiff_scale(bs.Lt, 1.5, n_diff=8)
    ref, br = O.dit_block(inp["x"], w, bs, inp["text_ctx"], inp["t_mod"], key_scale=g, gamma_o=1.5, return_branches=True)
    got = block_with_bf16_operands(inp["x"], w, bs, inp["text_ctx"], inp["t_mod"], key_scale=g, gamma_o=1.5)
    a, r = _errs(got, ref)
    da, dr = _errs(got - inp["x"], ref - inp["x"])
    print(f"[floor] stress={stress}: x max_abs={a:.3e} rel_l2={r:.3e}; delta rel_l2={dr:.3e}; max|ref|={np.abs(ref).max():.2f}")
    if not stress:
        # the benchmark's recipe: an order of magnitude inside the benchmark spec's bounds
        assert a < 2e-2 / 4 and r < 5e-3 / 4
        assert dr < 2e-2
    else:
        # the stress recipe: bf16 operands alone break max-abs 2e-2, and stay inside the scaled bound
        assert a > 2e-2
        assert a < np.abs(ref).max() * 2 ** -6 and r < 1e-2
        assert dr < 2e-2
