"""GPU parity of the single operations the block is made of (GEMM + epilogues,
LayerNorm/modulate, RMSNorm + RoPE, V transpose, attention) against the oracle."""
import math

import numpy as np
import pytest
import torch

import synth
from oracle import chorus_oracle as O
import paper_2604_04451_amd as P
from paper_2604_04451_amd import binding as B
from gpu_util import DEV, check, dev_bf16, dev_f32, host, host_bf16

pytestmark = pytest.mark.gpu


# --------------------------------------------------------------------- GEMM

@pytest.mark.parametrize("M,N,K", [(1, 64, 64), (100, 768, 256), (257, 1536, 1536), (1000, 64, 1536),
                                   (4099, 4608, 1536), (3000, 1536, 8960), (513, 1024, 64), (70, 8, 128),
                                   (4452, 4096, 512)])
def test_gemm_epilogues(M, N, K):
    """Every tile kernel (1: 128 x 64, 2: 256 x 128, 3: 256 x 256 and 4: 128 x 128 direct to LDS) and the automatic choice (0), each on
    every shape: tiles with ragged rows and columns, a single row, fewer columns than a tile has, K of one and of
    many steps; the four epilogues. At 4452 x 4096 x 512 the automatic choice cuts the rows: 4096 of them (one whole
    round of 256 x 256 tiles) in one launch, the other 356 on the 128 x 64 kernel in a second."""
    A = synth.round_bf16(synth.normal(M, "g.A", (M, K)))
    W = synth.round_bf16(synth.normal(M, "g.W", (N, K), 0.05))
    bias = synth.normal(M, "g.b", (N,), 0.5)
    g0 = synth.normal(M, "g.g0", (N,), 0.5)
    g1 = synth.normal(M, "g.g1", (N,), 0.5)
    resid = synth.normal(M, "g.r", (M, N))
    ref = O.linear(A, W, bias)
    ref0 = O.linear(A, W, np.zeros(N))
    gref = O.gelu_tanh(ref)
    dA, dW, db = dev_bf16(A), dev_bf16(W), dev_f32(bias)
    for kern in (0, 1, 2, 3, 4):
        print(f"[case] gemm M={M} N={N} K={K} kernel={kern}", flush=True)
        out = torch.empty(M, N, dtype=torch.bfloat16, device=DEV)
        B.chorus_gemm_bf16(dA, dW, B.EPI_BF16, out, db, kernel=kern)
        check(host_bf16(out), ref, f"gemm bf16 k{kern}", max_abs=np.abs(ref).max() * 2 ** -8, rel_l2=3e-3)
        B.chorus_gemm_bf16(dA, dW, B.EPI_GELU_BF16, out, db, kernel=kern)
        check(host_bf16(out), gref, f"gemm gelu k{kern}", max_abs=max(np.abs(gref).max() * 2 ** -8, 1e-3), rel_l2=3e-3)
        o32 = torch.empty(M, N, dtype=torch.float32, device=DEV)
        B.chorus_gemm_bf16(dA, dW, B.EPI_F32, o32, None, kernel=kern)
        check(host(o32), ref0, f"gemm f32 k{kern}", max_abs=1e-3, rel_l2=1e-5)
        r = dev_f32(resid)
        B.chorus_gemm_bf16(dA, dW, B.EPI_RESID, r, db, dev_f32(g0), dev_f32(g1), 1.0, kernel=kern)
        check(host(r), resid + (g0.astype(np.float64) + g1) * ref, f"gemm resid gated k{kern}", max_abs=1e-3, rel_l2=1e-5)
        r = dev_f32(resid)
        B.chorus_gemm_bf16(dA, dW, B.EPI_RESID, r, db, None, None, 1.5, kernel=kern)
        check(host(r), resid + 1.5 * ref, f"gemm resid scale k{kern}", max_abs=1e-3, rel_l2=1e-5)


# ------------------------------------------------------------- LN + modulate

@pytest.mark.parametrize("L,D", [(1, 256), (301, 256), (130, 1536), (37, 5120), (50, 320)])
def test_ln_modulate(L, D):
    print(f"[case] ln_modulate L={L} D={D}", flush=True)
    x = synth.normal(D, "ln.x", (L, D), 1.3, 0.4)
    tab = synth.normal(D, "ln.tab", (4, D), 0.3)
    out = torch.empty(L, D, dtype=torch.bfloat16, device=DEV)
    d = [dev_f32(tab[i]) for i in range(4)]
    B.chorus_ln_modulate(dev_f32(x), out, d[0], d[1], d[2], d[3], True)
    ref = O.layernorm(x) * (1.0 + tab[0].astype(np.float64) + tab[1]) + (tab[2].astype(np.float64) + tab[3])
    check(host_bf16(out), ref, "adaln", max_abs=np.abs(ref).max() * 2 ** -8, rel_l2=2.5e-3)
    B.chorus_ln_modulate(dev_f32(x), out, d[0], None, d[2], None, False)
    ref = O.layernorm(x) * tab[0].astype(np.float64) + tab[2]
    check(host_bf16(out), ref, "ln affine", max_abs=np.abs(ref).max() * 2 ** -8, rel_l2=2.5e-3)


# ------------------------------------------------------------ RMSNorm + RoPE

@pytest.mark.parametrize("H,dh,grid", [(4, 64, (4, 8, 8)), (12, 128, (5, 12, 20)), (2, 128, (21, 30, 52))])
def test_qk_norm_rope(H, dh, grid):
    print(f"[case] qk_norm_rope H={H} dh={dh} grid={grid}", flush=True)
    D = H * dh
    Ltok = grid[0] * grid[1] * grid[2]
    m = synth.bernoulli_mask(Ltok, 0.3, seed=dh) if Ltok > 2000 else np.ones(Ltok, np.uint8)
    idx = O.region_compact(m)
    L = idx.size
    Lpad = (L + 255) // 256 * 256
    z = synth.round_bf16(synth.normal(dh, "qk.z", (L, 3 * D), 1.5))
    gain = synth.normal(dh, "qk.g", (D,), 0.2, 1.5)
    out = torch.full((H, Lpad, dh), 3.0, dtype=torch.bfloat16, device=DEV)
    B.chorus_qk_norm_rope(dev_bf16(z), D, dev_f32(gain), out, L, H, dh,
                          torch.from_numpy(idx.astype(np.int32)).to(DEV), grid, True)
    ref = O.rope3d(O.rmsnorm(z[:, D:2 * D], gain), idx, grid, H, dh).reshape(L, H, dh).transpose(1, 0, 2)
    got = host_bf16(out)
    check(got[:, :L], ref, "rms+rope", max_abs=np.abs(ref).max() * 2 ** -8, rel_l2=2.5e-3)
    assert (got[:, L:] == 0).all()
    # no RoPE, identity positions
    B.chorus_qk_norm_rope(dev_bf16(z), 0, dev_f32(gain), out, L, H, dh, None, grid, False)
    ref = O.rmsnorm(z[:, :D], gain).reshape(L, H, dh).transpose(1, 0, 2)
    check(host_bf16(out)[:, :L], ref, "rms only", max_abs=np.abs(ref).max() * 2 ** -8, rel_l2=2.5e-3)
    # with an output factor (the pre-scaled queries of the long self-attention kernel): the same values times the factor
    c = float(np.log2(np.e) / np.sqrt(dh))
    B.chorus_qk_norm_rope(dev_bf16(z), 0, dev_f32(gain), out, L, H, dh, None, grid, False, c)
    check(host_bf16(out)[:, :L], ref * c, "rms only, scaled", max_abs=np.abs(ref).max() * c * 2 ** -8, rel_l2=2.5e-3)
    with pytest.raises(P.ChorusError):
        B.chorus_qk_norm_rope(dev_bf16(z), 0, dev_f32(gain), out, L, H, dh, None, grid, False, 0.0)


def _vt_reference(v, Lpad):
    """[L, D] -> [D, Lpad] with the 16-group token permutation position 8c+4u+i <- token 8u+4c+i."""
    L, D = v.shape
    vp = np.zeros((Lpad, D), v.dtype)
    vp[:L] = v
    pos = np.arange(Lpad)
    G, r = pos // 16, pos % 16
    c, u, i = r // 8, (r // 4) % 2, r % 4
    tok = 16 * G + 8 * u + 4 * c + i
    return vp[tok].T.copy()


@pytest.mark.parametrize("L,D", [(1, 64), (100, 256), (1200, 1536)])
def test_v_transpose_bit_exact(L, D):
    print(f"[case] v_transpose L={L} D={D}", flush=True)
    Lpad = (L + 255) // 256 * 256
    z = synth.round_bf16(synth.normal(L, "vt.z", (L, 3 * D)))
    out = torch.full((D, Lpad), 5.0, dtype=torch.bfloat16, device=DEV)
    B.chorus_v_transpose(dev_bf16(z), 2 * D, out, L)
    np.testing.assert_array_equal(host_bf16(out), _vt_reference(z[:, 2 * D:].astype(np.float64), Lpad))


# ---------------------------------------------------------------- attention

def _attn_case(H, dh, Lq, Lk, variant, col_scale=None, q_std=1.0, seed=0, name="", expect_tiles=None):
    """One attention launch against the oracle. Keys are padded to 128 for the default choice and the 128-key
    tile kernel (what the block does: it pads rows to 256), to 64 for the 64-key one."""
    D = H * dh
    q = synth.normal(seed, "at.q", (Lq, D), q_std)
    if variant == 6:
        # the kernel is handed bf16(q * c); the oracle gets those same rounded queries with the factor taken out again
        c = np.float32(np.log2(np.e) / np.sqrt(dh))
        q_dev = synth.round_bf16(q * c)
        q = q_dev.astype(np.float64) / np.float64(c)
    else:
        q = q_dev = synth.round_bf16(q)
    k = synth.round_bf16(synth.normal(seed, "at.k", (Lk, D), q_std))
    v = synth.round_bf16(synth.normal(seed, "at.v", (Lk, D)))
    LqPad = (Lq + 255) // 256 * 256
    kpad = 64 if variant == 3 else 128
    LkPad = (Lk + kpad - 1) // kpad * kpad
    Q = torch.zeros(H, LqPad, dh, dtype=torch.bfloat16, device=DEV)
    K = torch.zeros(H, LkPad, dh, dtype=torch.bfloat16, device=DEV)
    Q[:, :Lq] = dev_bf16(q_dev).reshape(Lq, H, dh).transpose(0, 1)
    K[:, :Lk] = dev_bf16(k).reshape(Lk, H, dh).transpose(0, 1)
    Vt = torch.from_numpy(synth.to_bf16_bits(_vt_reference(v, LkPad).astype(np.float32)).reshape(D, LkPad).view(np.int16)).to(DEV).view(torch.bfloat16)
    Oo = torch.full((Lq, D), 9.0, dtype=torch.bfloat16, device=DEV)
    cs = None if col_scale is None else dev_f32(col_scale)
    B.chorus_attention(Q, K, Vt, Oo, cs, Lq, Lk, variant)
    ref = O.attention(np.asarray(q, np.float64), O.tgaa_amplify_keys(k.astype(np.float64), col_scale), v.astype(np.float64), H, dh)
    return check(host_bf16(Oo), ref, f"attention {name} H={H} dh={dh} Lq={Lq} Lk={Lk} v{variant}",
                 max_abs=max(np.abs(ref).max() * 2 ** -7, 2e-3), rel_l2=5e-3)


# variant 0 is the library's own choice (128-key tiles from 512 keys on, else 64-key tiles), 3 and 5 force the
# 64-key and the 128-key 16x16x32-MFMA tile kernel, 6 is the latter fed with pre-scaled queries (what
# the block launches for long self-attention): every shape runs through the kernel the block and the benchmark launch.
ATTN_VARIANTS = [0, 3, 5, 6]


@pytest.mark.parametrize("variant", ATTN_VARIANTS)
@pytest.mark.parametrize("H,dh,Lq,Lk", [(2, 64, 300, 300), (3, 128, 500, 333), (1, 128, 1, 1), (2, 128, 64, 64),
                                        (2, 64, 257, 65), (12, 128, 1200, 1200), (4, 64, 256, 16),
                                        (2, 128, 300, 2048), (2, 128, 513, 2049), (3, 64, 300, 2049),
                                        (1, 128, 260, 2176 + 127), (1, 64, 40, 129)])
def test_attention_plain(H, dh, Lq, Lk, variant):
    print(f"[case] attention H={H} dh={dh} Lq={Lq} Lk={Lk} variant={variant}", flush=True)
    _attn_case(H, dh, Lq, Lk, variant, name="plain")


@pytest.mark.parametrize("variant", ATTN_VARIANTS)
def test_attention_peaked(variant):
    """Logits with std ~4: rows dominated by few keys; catches masking / rescale mistakes that
    near-uniform rows (output ~ mean V) would hide. Key counts with tails of 4, 16, 1 and 81 keys in the
    last 128-key tile, above and below 512 and 2048 keys (the default switches tile size at 512)."""
    print(f"[case] attention peaked variant={variant}", flush=True)
    _attn_case(4, 128, 700, 900, variant, q_std=2.0, seed=3, name="peaked")
    _attn_case(2, 64, 333, 2000, variant, q_std=2.0, seed=4, name="peaked64")
    _attn_case(2, 128, 600, 2049, variant, q_std=2.0, seed=5, name="peaked 2049")
    _attn_case(2, 64, 300, 2385, variant, q_std=2.0, seed=6, name="peaked64 2385")
    _attn_case(1, 128, 257, 4096, variant, q_std=2.5, seed=8, name="peaked 4096 no tail")


def test_attention_variant_argument_errors():
    """Unknown variants, a column scale off a 16-byte boundary and 64-key padding with the 128-key kernel are refused."""
    H, dh, L = 1, 128, 128
    Q = torch.zeros(H, 256, dh, dtype=torch.bfloat16, device=DEV)
    K = torch.zeros(H, 128, dh, dtype=torch.bfloat16, device=DEV)
    Vt = torch.zeros(H * dh, 128, dtype=torch.bfloat16, device=DEV)
    Oo = torch.zeros(L, H * dh, dtype=torch.bfloat16, device=DEV)
    unaligned = torch.ones(L + 4, device=DEV)[1:L + 1]  # a column scale must sit on a 16-byte boundary
    for v in (0, 3, 5, 6):
        with pytest.raises(P.ChorusError):
            B.chorus_attention(Q, K, Vt, Oo, unaligned, L, L, v)
    for bad in (1, 2, 4, 7, -1):
        with pytest.raises(P.ChorusError):
            B.chorus_attention(Q, K, Vt, Oo, None, L, L, bad)
    K64 = torch.zeros(H, 64, dh, dtype=torch.bfloat16, device=DEV)
    Vt64 = torch.zeros(H * dh, 64, dtype=torch.bfloat16, device=DEV)
    for v in (5, 6):
        with pytest.raises(P.ChorusError):
            B.chorus_attention(Q, K64, Vt64, Oo, None, L, 64, v)


@pytest.mark.parametrize("variant", [0, 3, 5, 6])
@pytest.mark.parametrize("H,dh,Lq,Lt", [(4, 64, 256, 16), (12, 128, 700, 512), (2, 128, 100, 77), (2, 128, 300, 700),
                                        (1, 64, 260, 1027)])
def test_attention_tgaa_column_scale(H, dh, Lq, Lt, variant):
    """Eq. 2 as a per-key logit factor, on the 64-key kernel (3), on the 16x16x32 kernel with and without pre-scaled
    queries (5, 6) and on the default choice (0: the latter from 512 keys on); key counts that end a 128-key tile
    on a multiple of four and off one."""
    print(f"[case] cross-attention TGAA H={H} dh={dh} Lq={Lq} Lt={Lt} variant={variant}", flush=True)
    _attn_case(H, dh, Lq, Lt, variant, col_scale=synth.tdiff_scale(Lt, 1.5), q_std=1.5, name="tgaa-all")
    _attn_case(H, dh, Lq, Lt, variant, col_scale=synth.tdiff_scale(Lt, 1.5, n_diff=max(1, Lt // 64)), q_std=1.5, name="tgaa-subset")
    # neutral scale equals the plain kernel's result
    a = _attn_case(H, dh, Lq, Lt, variant, col_scale=np.ones(Lt, np.float32), q_std=1.5, name="tgaa-neutral")
    b = _attn_case(H, dh, Lq, Lt, variant, col_scale=None, q_std=1.5, name="plain")
    assert abs(a[1] - b[1]) < 1e-3


def test_mfma_ceiling_runs_and_orders():
    """The benchmark diagnostic: a bare MFMA loop. Constant operands sustain more than random ones, and
    LDS operand reads plus exponentials cost throughput; all within the part's nominal 2.5 PFLOP/s."""
    print("[case] mfma_ceiling", flush=True)
    ones = B.chorus_mfma_ceiling(False, 0, 5)
    rnd = B.chorus_mfma_ceiling(True, 0, 5)
    mix = B.chorus_mfma_ceiling(True, 3, 5)
    print(f"[info] mfma ceiling TFLOP/s: ones {ones:.0f}, normal {rnd:.0f}, normal + LDS operand + exp2 {mix:.0f}", flush=True)
    assert 300.0 < mix < rnd * 1.02 and rnd < ones * 1.02 and ones < 2700.0


@pytest.mark.parametrize("name,freq_dim", [("c1", 256), ("wan1p3b_small", 256), ("c1", 64)])
def test_time_mod(name, freq_dim):
    print(f"[case] time_mod {name} freq_dim={freq_dim}", flush=True)
    bs = synth.SHAPES[name]
    tw = synth.time_weights(bs, 0, freq_dim=freq_dim)
    dtw = B.DeviceTime(tw)
    for t in (0.0, 1.0, 421.5, 999.0):
        t_mod, t_head = B.chorus_time_mod(t, dtw)
        rm, rh = O.time_mod(float(np.float32(t)), tw, bs.D, freq_dim)
        # fp32 sincos of arguments up to 1000 rad, then three fp32 matrix-vector products
        check(host(t_mod), rm, f"t_mod t={t}", max_abs=2e-4 * max(1.0, np.abs(rm).max()), rel_l2=2e-4)
        check(host(t_head), rh, f"t_head t={t}", max_abs=2e-4 * max(1.0, np.abs(rh).max()), rel_l2=2e-4)
        assert torch.equal(t_head[0], t_head[1])
