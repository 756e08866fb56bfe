"""Parity at the benchmark's full sizes (Wan2.1-1.3B-shaped 480p: 32760 tokens, D 1536,
12 x 128 heads, F 8960, 512 text tokens), in the launch configuration bench.py times.
The oracle cannot run a whole block here in seconds, so it is teacher-forced on the
block's input and computes a seeded sample of output rows exactly (each sampled row still
attends to all keys)."""
import numpy as np
import pytest
import torch

import synth
from oracle import chorus_oracle as O
import paper_2604_04451_amd as P
from paper_2604_04451_amd import binding as B
from gpu_util import DEV, check, dev_bf16, dev_f32, errs, host, host_bf16
from test_gpu_ops import _vt_reference

pytestmark = pytest.mark.gpu


def _rows(L, n, seed):
    r = synth.stream(seed, "rows").permutation(L)[:n]
    return np.unique(np.concatenate([r, [0, L - 1, L - 2, (L // 256) * 256, (L // 256) * 256 - 1]]))


# (heads, tokens): the full-step and the 40 % stage-2 token counts of the 480p workload in the benchmark's head
# count, and the 720p token count of the 14B-shaped workload on two heads (the oracle rows cost 4 L dh each).
# Tails of the last key tile: 32760 = 255 x 128 + 120 = 511 x 64 + 56; 13104 = 102 x 128 + 48 = 204 x 64 + 48;
# 75600 = 590 x 128 + 80 = 1181 x 64 + 16.
@pytest.mark.parametrize("H,L", [(12, 32760), (12, 13104), (2, 75600)])
def test_self_attention_full_length_peaked(H, L):
    """Self-attention at the benchmark's own lengths with peaked logits (std ~4), sampled query rows against
    the oracle: the library's default choice (the 128-key tile kernel the benchmark times) and both tile sizes
    forced."""
    dh = 128
    print(f"[case] attention full length H={H} L={L}", flush=True)
    D = H * dh
    q = synth.round_bf16(synth.normal(7, "fa.q", (L, D), 2.0))
    k = synth.round_bf16(synth.normal(7, "fa.k", (L, D), 2.0))
    v = synth.round_bf16(synth.normal(7, "fa.v", (L, D)))
    Lpad = (L + 255) // 256 * 256
    Q = torch.zeros(H, Lpad, dh, dtype=torch.bfloat16, device=DEV)
    K = torch.zeros(H, Lpad, dh, dtype=torch.bfloat16, device=DEV)
    Q[:, :L] = dev_bf16(q).reshape(L, H, dh).transpose(0, 1)
    K[:, :L] = dev_bf16(k).reshape(L, H, dh).transpose(0, 1)
    Vt = torch.empty(D, Lpad, dtype=torch.bfloat16, device=DEV)
    B.chorus_v_transpose(dev_bf16(v), 0, Vt, L)
    rows = _rows(L, 96, 7)
    ref = O.attention(q[rows].astype(np.float64), k.astype(np.float64), v.astype(np.float64), H, dh)
    for variant in (0, 4, 3):
        print(f"[launch] attention full length H={H} L={L} variant={variant}", flush=True)
        Oo = torch.empty(L, D, dtype=torch.bfloat16, device=DEV)
        B.chorus_attention(Q, K, Vt, Oo, None, L, L, variant)
        got = host_bf16(Oo)
        assert np.isfinite(got).all()
        check(got[rows], ref, f"attention full length H={H} L={L} v{variant}", max_abs=max(np.abs(ref).max() * 2 ** -7, 2e-3), rel_l2=5e-3)


@pytest.mark.parametrize("masked", [False, True, "bernoulli"])
def test_block_full_shape_row_sampled(masked):
    bs = synth.SHAPES["wan1p3b_480p"]
    print(f"[case] block 1.3B 480p full shape masked={masked}", flush=True)
    w = synth.block_weights(bs, 0)
    inp = synth.block_inputs(bs, 0)
    g = synth.tdiff_scale(bs.Lt, 1.5, n_diff=8) if masked else None
    go = 1.5 if masked else 1.0
    if masked == "bernoulli":
        mask = synth.bernoulli_mask(bs.L, 0.5, seed=0)           # region sweep: i.i.d. per-token mask
        idx = O.region_compact(mask)
    elif masked:
        mask = synth.box_mask(bs.grid, 21, 24, 26, 0, 3, 13)     # exactly 40% of the tokens
        idx = O.region_compact(mask)
        assert idx.size == 13104
    else:
        idx = np.arange(bs.L)
    x_in = inp["x"][idx]
    shape = P.make_block_shape(bs.D, bs.H, bs.dh, bs.F, bs.Lt, bs.grid)
    dw = P.upload_block_weights(w)
    x = dev_f32(x_in)
    tidx = torch.from_numpy(idx.astype(np.int32)).to(DEV) if masked else None
    P.chorus_dit_block_step(shape, dw, x, idx.size, tidx, dev_bf16(inp["text_ctx"]), dev_f32(inp["t_mod"]),
                            None if g is None else dev_f32(g), go)
    got = host(x)
    assert np.isfinite(got).all()
    rows = _rows(idx.size, 48, 11)
    print(f"[oracle] {rows.size} sampled rows of {idx.size}", flush=True)
    ref = O.dit_block(x_in, w, bs, inp["text_ctx"], inp["t_mod"], token_idx=idx, key_scale=g, gamma_o=go, rows=rows)
    check(got[rows], ref, f"block full shape masked={masked} x")
    a, r = errs(got[rows] - x_in[rows], ref - x_in[rows])
    print(f"[parity] block full shape masked={masked} delta: max_abs={a:.3e} rel_l2={r:.3e}", flush=True)
    assert r <= 2e-2
    # rows outside the sample: finite and changed
    assert np.abs(got - x_in).max() > 1e-3
