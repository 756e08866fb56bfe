"""CPU oracle for the Chorus hot path. TEST INFRASTRUCTURE ONLY.

Plain numpy, float64 throughout, written from the paper's definitions. Nothing
here is blocked, fused or reordered; numpy matmul / argmax / tanh serve as steps.
Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
module; the product path never does, and this module imports nothing from it.

What the paper fixes and what it leaves open
--------------------------------------------
* Stage-1 retrieval (Sec. 3.1, "Full Reuse"): top-1 cosine similarity against the
  cached prompt embeddings, a hit when the score reaches the threshold tau
  (the formal fallback rule is m < tau => K1 = K2 = 0, Sec. 3.1 "Stage Boundary
  Determination").
* Stage boundaries (Eq. 1) and the TGAA decay (Eq. 4): the paper gives only
  properties (monotone in m, 0 <= K1 <= K2 <= N, factors >= 1, decreasing in step
  and in m). `denoise_schedule` is one concrete map with those properties; its
  VALUES are "parity unpinned" against the paper, its properties are tested.
* TGAA key amplification (Eq. 2) and output amplification (Eq. 3): implemented
  literally (K' built by scaling the selected key rows).
* Hierarchical masks and latent fusion (Eq. 5, Eq. 6): fusion is implemented as
  written, M*L + (1-M)*SL with a binary M.
* The DiT block itself is only drawn (Fig. 2) and described in prose (Sec. 2.1):
  self-attention, cross-attention on the prompt, timestep injection, FFN. Its
  arithmetic here is the Wan2.1-shaped block the benchmark configurations name
  (AdaLN modulation, RMSNorm on q/k, 3-D RoPE, tanh-GELU FFN); each choice is
  stated at the function that makes it.
* Cache update (Sec. 3.1): `cache_insert`; several stored depths per entry enter the schedule as
  `stored_steps` (K1 snaps to a stored depth). `cache_lookup_topk` is the batched retrieval with
  candidates; its column 0 is `cache_lookup`.
* Low-precision storage of the cached embeddings (bf16 / FP8 E4M3) with an exact re-rank:
  `cache_lowprec_encode`, `cache_lookup_lowprec`; its result is `cache_lookup`'s by construction.
* Timestep injection (Sec. 2.1, Fig. 2): `time_mod`, Wan2.1-shaped like the block.
* The sampler (Sec. 4.1: DPM++ with default settings, no formulas given): the published
  DPM-Solver++ multistep update of order <= 2 in data-prediction form on the rectified-flow
  path, plus classifier-free guidance for the models that use it. The Euler update of
  `denoise_step` is its first-order case.
"""
from __future__ import annotations

import math

import numpy as np

F64 = np.float64

# --------------------------------------------------------------------------
# Stage-1 retrieval (Sec. 3.1 "Full Reuse"; appendix: cosine top-1 over the cache)
# --------------------------------------------------------------------------


def cosine_scores(cache_emb, query):
    """s_j = <q, c_j> / (|q| |c_j|); a zero-norm vector scores -inf."""
    c = np.asarray(cache_emb, F64)
    q = np.asarray(query, F64)
    if c.shape[0] == 0:
        return np.zeros(0, F64)
    dots = c @ q
    nq = math.sqrt(float(q @ q))
    nc = np.sqrt(np.einsum("ij,ij->i", c, c))
    denom = nq * nc
    s = np.full(c.shape[0], -np.inf, F64)
    ok = denom > 0
    s[ok] = dots[ok] / denom[ok]
    return s


def cache_lookup(cache_emb, query, tau):
    """Returns (index, score m, hit). Lowest index wins ties; empty cache is a miss
    with index -1 and score -inf."""
    s = cosine_scores(cache_emb, query)
    if s.size == 0:
        return -1, -math.inf, False
    j = int(np.argmax(s))  # numpy returns the first maximum
    m = float(s[j])
    return j, m, bool(m >= tau)


# --------------------------------------------------------------------------
# Low-precision embedding storage with an exact re-rank (cache maintenance around the
# retrieval of Sec. 3.1 "Full Reuse"; the paper's cache backend is a vector store, appendix).
# The result is DEFINED to be `cache_lookup`'s: the low-precision copy only decides which rows
# are re-scored from the fp32 rows. Encodings are written from the published formats
# (bfloat16: 1 sign, 8 exponent, 7 fraction bits, fp32's exponent range; OCP FP8 E4M3:
# 1 sign, 4 exponent bits with bias 7, 3 fraction bits, subnormals, largest finite 448, no
# infinities), both with round-to-nearest-even.
# --------------------------------------------------------------------------

def bf16_encode(x):
    """float32 values -> bf16 bit patterns (uint16), round to nearest, ties to even."""
    bits = np.ascontiguousarray(x, np.float32).view(np.uint32).astype(np.uint64)
    lsb = (bits >> np.uint64(16)) & np.uint64(1)
    return ((bits + np.uint64(0x7FFF) + lsb) >> np.uint64(16)).astype(np.uint16)


def bf16_decode(code):
    return (np.asarray(code, np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(F64)


def fp8_e4m3_decode(code):
    """OCP FP8 E4M3 bit patterns -> values: (-1)^s 2^(e-7) (1 + f/8) for e > 0, (-1)^s 2^-6 (f/8) for e = 0."""
    c = np.asarray(code, np.uint8).astype(np.int64)
    sgn = np.where(c & 0x80, -1.0, 1.0)
    e = (c >> 3) & 0xF
    f = c & 0x7
    mag = np.where(e > 0, np.ldexp(1.0 + f / 8.0, e - 7), np.ldexp(f / 8.0, -6))
    return sgn * mag


def fp8_e4m3_encode(y):
    """Finite values -> OCP FP8 E4M3 bit patterns: the nearest representable magnitude (ties to the even
    code), magnitudes beyond 448 saturate to 448. Written as a search over the 127 finite magnitudes."""
    y = np.asarray(y, F64)
    mags = fp8_e4m3_decode(np.arange(127, dtype=np.uint8))          # codes 0x00..0x7E, ascending
    a = np.minimum(np.abs(y), 448.0)
    hi = np.searchsorted(mags, a, side="left").clip(0, 126)         # first magnitude >= a
    lo = np.maximum(hi - 1, 0)
    d_hi, d_lo = mags[hi] - a, a - mags[lo]
    pick_lo = (d_lo < d_hi) | ((d_lo == d_hi) & (lo % 2 == 0))
    code = np.where(pick_lo, lo, hi).astype(np.uint8)
    return np.where(np.signbit(y), code | np.uint8(0x80), code).astype(np.uint8)


LOWPREC_FORMATS = ("bf16", "fp8")


def cache_lowprec_encode(cache_emb, fmt):
    """The low-precision copy of the cached prompt embeddings. bf16: every element rounded. fp8: every row is
    first scaled so that its largest magnitude maps to 448 (inv = 448 / max|c| and y = c * inv, both single fp32
    operations, the precision in which the integer code is decided), then rounded; an all-zero row encodes as zeros.
    The scale is not kept: cosine similarity does not depend on it."""
    c = np.ascontiguousarray(cache_emb, np.float32)
    if fmt == "bf16":
        return bf16_encode(c)
    assert fmt == "fp8"
    amax = np.abs(c).max(axis=1, keepdims=True) if c.shape[0] else np.zeros((0, 1), np.float32)
    with np.errstate(divide="ignore"):
        inv = np.where(amax > 0, np.float32(448.0) / amax, np.float32(0.0)).astype(np.float32)
    return fp8_e4m3_encode((c * inv).astype(np.float32))


def cache_lowprec_decode(codes, fmt):
    return bf16_decode(codes) if fmt == "bf16" else fp8_e4m3_decode(codes)


def lowprec_margin(fmt, d):
    """Twice the largest change of a cosine score when a row c is replaced by its low-precision copy c^:
    |cos(q, c^) - cos(q, c)| <= angle(c, c^) <= asin(|c^ - c| / |c|). bf16 keeps 8 significant bits: every element
    moves by at most 2^-8 of itself. FP8 E4M3 keeps 4 (2^-4 of itself) down to 2^-6, below that the step is 2^-9
    (at most 2^-10 off), and the scaled row's norm is at least 448."""
    delta = 2.0 ** -8 if fmt == "bf16" else 2.0 ** -4 + math.sqrt(d) * 2.0 ** -10 / 448.0
    return 2.0 * math.asin(delta)


def cache_lookup_lowprec(cache_emb, codes, fmt, query, tau, margin=None):
    """Two-stage retrieval: score every row from its low-precision copy, keep the rows within `margin` of the best
    approximate score, re-score those from the fp32 rows and take the best (lowest index among equal scores).
    With margin >= lowprec_margin the true best row is always among the candidates, so (index, score, hit) are
    `cache_lookup`'s. Returns (index, score, hit, number of re-scored rows)."""
    c = np.asarray(cache_emb, F64)
    if c.shape[0] == 0:
        return -1, -math.inf, False, 0
    if margin is None:
        margin = lowprec_margin(fmt, c.shape[1])
    approx = cosine_scores(cache_lowprec_decode(codes, fmt), query)
    best = approx.max()
    if not np.isfinite(best):                     # zero-norm query or all rows zero: every exact score is -inf too
        return 0, -math.inf, False, 0
    cand = np.nonzero(approx >= best - margin)[0]
    exact = cosine_scores(c[cand], query)
    k = int(np.argmax(exact))
    m = float(exact[k])
    return int(cand[k]), m, bool(m >= tau), int(cand.size)


# --------------------------------------------------------------------------
# Stage boundaries and TGAA decay (Eq. 1, Eq. 4) -- values parity unpinned
# --------------------------------------------------------------------------

DEFAULT_SCHED = dict(a1=0.25, b1=0.25, a2=0.25, b2=0.25, r3=1, Gamma_k=1.5, Gamma_o=1.5, lam=0.5,
                     gamma_override=0.0)


def cache_lookup_topk(cache_emb, queries, tau, k):
    """The k best entries for each of several prompt embeddings (the retrieval of Sec. 3.1 for a
    batch of queued requests; k > 1 gives the scheduler candidates to choose from).
    Returns (index [Q, k], score [Q, k], hit [Q]): entries by descending cosine, equal scores by
    ascending index; positions beyond the cache size hold index -1 and score -inf;
    hit[q] = score[q, 0] >= tau. Column 0 is `cache_lookup` of that query."""
    queries = np.asarray(queries, F64)
    Q = queries.shape[0]
    k = int(k)
    idx = np.full((Q, k), -1, np.int64)
    sc = np.full((Q, k), -np.inf, F64)
    hit = np.zeros(Q, bool)
    for qi in range(Q):
        s = cosine_scores(cache_emb, queries[qi])
        order = sorted(range(s.size), key=lambda j: (-s[j], j))[:k]
        for r, j in enumerate(order):
            idx[qi, r] = j
            sc[qi, r] = s[j]
        hit[qi] = bool(sc[qi, 0] >= tau) if k > 0 else False
    return idx, sc, hit


def cache_insert(cache_emb, cache_latents, slot, emb, latent):
    """Cache update (Sec. 3.1 "Cache Update"): after a miss the request's prompt embedding and an
    intermediate latent are stored for later requests. Which entry is replaced is the caller's
    policy (the paper names none). Returns new arrays; the inputs are left untouched."""
    ce = np.array(cache_emb, copy=True)
    cl = np.array(cache_latents, copy=True)
    assert 0 <= slot < ce.shape[0] == cl.shape[0]
    ce[slot] = np.asarray(emb, ce.dtype)
    cl[slot] = np.asarray(latent, cl.dtype).reshape(cl.shape[1:])
    return ce, cl


def denoise_schedule(m, tau, N, params=None, stored_steps=None):
    """(K1, K2, plan) with plan[i] = (stage, gamma_k, gamma_o) for step i (0-based).

    stored_steps (optional): the depths k at which the matched entry holds an intermediate
    latent (the state after k steps; Sec. 3.1 "Cache Update" keeps several). Full reuse can
    only resume from a stored state, so K1 becomes the largest stored depth not above the
    K1 of Eq. 1; with none the request has no usable source latent and runs as a miss.
    The stage-2 length K2 - K1 is kept.

    m < tau  =>  K1 = K2 = 0 and every step is a plain stage-3 step.
    Otherwise s = clip((m - tau)/(1 - tau), 0, 1) and
      K1 = clip(floor(N (a1 + b1 s) + 1e-9), 0, N - r3)
      K2 = clip(K1 + floor(N (a2 + b2 s) + 1e-9), K1, N - r3)
    so both grow with m and at least r3 steps stay full compute (Sec. 1: the last
    stage always recomputes everything).
    For a computed step i >= K1:  w = max(0, 1 - (i - K1)/max(1, K2 - K1)),
      gamma = max(1, 1 + (Gamma - 1)(1 - lam s) w)
    which decreases with the step, decreases with m and never drops below 1
    (the three principles under Eq. 4). Reused steps (i < K1) run no attention; their
    factors are reported as 1. gamma_override > 0 replaces the factors of the
    stage-2 steps by that constant.
    """
    p = dict(DEFAULT_SCHED)
    if params:
        p.update(params)
    N = int(N)
    if not (m >= tau):  # also catches NaN and -inf
        return 0, 0, [(3, 1.0, 1.0) for _ in range(N)]
    s = min(max((float(m) - tau) / (1.0 - tau), 0.0), 1.0) if tau < 1.0 else 1.0
    hi = max(N - int(p["r3"]), 0)
    K1 = min(max(int(math.floor(N * (p["a1"] + p["b1"] * s) + 1e-9)), 0), hi)
    if stored_steps is not None:
        usable = [int(k) for k in stored_steps if 1 <= int(k) <= K1]
        if not usable:
            return 0, 0, [(3, 1.0, 1.0) for _ in range(N)]
        K1 = max(usable)
    K2 = min(max(K1 + int(math.floor(N * (p["a2"] + p["b2"] * s) + 1e-9)), K1), hi)
    plan = []
    for i in range(N):
        if i < K1:
            plan.append((1, 1.0, 1.0))
            continue
        stage = 2 if i < K2 else 3
        w = max(0.0, 1.0 - (i - K1) / max(1, K2 - K1))
        gk = max(1.0, 1.0 + (p["Gamma_k"] - 1.0) * (1.0 - p["lam"] * s) * w)
        go = max(1.0, 1.0 + (p["Gamma_o"] - 1.0) * (1.0 - p["lam"] * s) * w)
        if stage == 2 and p["gamma_override"] > 0:
            gk = go = float(p["gamma_override"])
        plan.append((stage, gk, go))
    return K1, K2, plan


# --------------------------------------------------------------------------
# Pointwise pieces of the block
# --------------------------------------------------------------------------

LN_EPS = 1e-6


def layernorm(x, eps=LN_EPS):
    """LayerNorm over the last axis, no affine, biased variance."""
    x = np.asarray(x, F64)
    mu = x.mean(-1, keepdims=True)
    var = ((x - mu) ** 2).mean(-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps)


def rmsnorm(z, gain, eps=LN_EPS):
    """z / sqrt(mean(z^2) + eps) * gain over the whole last axis (all heads together)."""
    z = np.asarray(z, F64)
    return z / np.sqrt((z * z).mean(-1, keepdims=True) + eps) * np.asarray(gain, F64)


def gelu_tanh(x):
    x = np.asarray(x, F64)
    return 0.5 * x * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (x + 0.044715 * x ** 3)))


def linear(x, w, b):
    """y = x W^T + b with W stored [out, in]."""
    return np.asarray(x, F64) @ np.asarray(w, F64).T + np.asarray(b, F64)


def rope_group_sizes(dh):
    """Head dims are split into consecutive (t, h, w) groups."""
    s = dh // 6
    return dh - 4 * s, 2 * s, 2 * s


def token_positions(token_idx, grid):
    """Original token id n -> (t, h, w) on the token grid (T, Hg, Wg), row-major."""
    _, Hg, Wg = grid
    n = np.asarray(token_idx, np.int64)
    return n // (Hg * Wg), (n // Wg) % Hg, n % Wg


def rope3d(z, token_idx, grid, H, dh, theta=10000.0):
    """3-D rotary embedding on z [L, H*dh]. In a group of size g, the pair
    (2p, 2p+1) of every head rotates by pos * theta^(-2p/g), pos being the token's
    t, h or w coordinate for the first, second, third group."""
    z = np.asarray(z, F64)
    L = z.shape[0]
    zh = z.reshape(L, H, dh).copy()
    pos = token_positions(token_idx, grid)
    off = 0
    for g, pcoord in zip(rope_group_sizes(dh), pos):
        for p in range(g // 2):
            ang = pcoord.astype(F64) * theta ** (-2.0 * p / g)
            c, s = np.cos(ang)[:, None], np.sin(ang)[:, None]
            a = zh[:, :, off + 2 * p].copy()
            b = zh[:, :, off + 2 * p + 1].copy()
            zh[:, :, off + 2 * p] = a * c - b * s
            zh[:, :, off + 2 * p + 1] = a * s + b * c
        off += g
    return zh.reshape(L, H * dh)


def softmax_rows(logits):
    m = logits.max(-1, keepdims=True)
    e = np.exp(logits - m)
    return e / e.sum(-1, keepdims=True)


def attention(q, k, v, H, dh, return_probs=False):
    """softmax(q k^T / sqrt(dh)) v per head; q [Lq, H*dh], k, v [Lk, H*dh]."""
    Lq, Lk = q.shape[0], k.shape[0]
    qh = q.reshape(Lq, H, dh).transpose(1, 0, 2)
    kh = k.reshape(Lk, H, dh).transpose(1, 0, 2)
    vh = v.reshape(Lk, H, dh).transpose(1, 0, 2)
    out = np.empty((H, Lq, dh), F64)
    probs = []
    for h in range(H):
        p = softmax_rows(qh[h] @ kh[h].T / math.sqrt(dh))
        out[h] = p @ vh[h]
        if return_probs:
            probs.append(p)
    o = out.transpose(1, 0, 2).reshape(Lq, H * dh)
    return (o, probs) if return_probs else o


def tgaa_amplify_keys(k, key_scale):
    """Eq. 2, first line: K'[j, :] = g_j K[j, :] with g_j = gamma_k on the differential
    tokens and 1 elsewhere (key_scale is that per-token vector; None leaves K as is)."""
    if key_scale is None:
        return k
    return np.asarray(key_scale, F64)[:, None] * k


# --------------------------------------------------------------------------
# The DiT block (Sec. 2.1, Fig. 2; TGAA per Eq. 2 and Eq. 3)
# --------------------------------------------------------------------------


def dit_block(x, w, shape, text_ctx, t_mod, token_idx=None, key_scale=None, gamma_o=1.0,
              rows=None, return_branches=False):
    """One block forward on the rows of x [Ls, D]; returns the new x.

    shape: dict/obj with D, H, dh, grid. token_idx: original token ids of the rows
    (None = identity) -- they fix the RoPE positions, so a compacted subset keeps
    its true (t, h, w). Every row of x takes part as a key/value of self-attention:
    in stage 2 the caller passes only the selected tokens, which is the paper's
    "select the regions to be computed" (Sec. 3.3.3).

    e = mod_table + t_mod gives (shift, scale, gate) for the self-attention and FFN
    branches. The six steps:
      1. h = LN(x)(1 + scale_sa) + shift_sa;  q, k, v = linear(h)
      2. q, k RMS-normalised over the full width with learned gains
      3. 3-D RoPE on q, k
      4. x += gate_sa * linear_o(softmax(q k^T / sqrt(dh)) v)
      5. cross-attention on the text context with TGAA: queries from an affine
         LayerNorm of x, q/k RMS-normalised, keys amplified AFTER normalisation
         (Eq. 2; a scale applied before a per-token norm would cancel), and
         x += gamma_o * cross_attn(x) (Eq. 3, the bias of the output projection
         is part of cross_attn)
      6. x += gate_ffn * linear_2(gelu_tanh(linear_1(LN(x)(1 + scale_ffn) + shift_ffn)))

    rows: optional index array; then only those rows are carried through (their
    self-attention still sees all Ls keys) and [len(rows), D] is returned. This is
    the same arithmetic restricted to some output rows, used at sizes where a full
    block is out of reach.
    """
    D, H, dh = shape.D, shape.H, shape.dh
    grid = shape.grid
    x = np.asarray(x, F64)
    Ls = x.shape[0]
    if token_idx is None:
        token_idx = np.arange(Ls)
    token_idx = np.asarray(token_idx, np.int64)
    e = np.asarray(w["mod_table"], F64) + np.asarray(t_mod, F64)
    sh1, sc1, g1, sh2, sc2, g2 = e
    sel = np.arange(Ls) if rows is None else np.asarray(rows, np.int64)

    # 1-3: self-attention inputs
    h = layernorm(x) * (1.0 + sc1) + sh1
    wq, wk, wv = (np.asarray(w["w_qkv"], F64)[i * D:(i + 1) * D] for i in range(3))
    bq, bk, bv = (np.asarray(w["b_qkv"], F64)[i * D:(i + 1) * D] for i in range(3))
    q = rope3d(rmsnorm(linear(h[sel], wq, bq), w["g_q"]), token_idx[sel], grid, H, dh)
    k = rope3d(rmsnorm(linear(h, wk, bk), w["g_k"]), token_idx, grid, H, dh)
    v = linear(h, wv, bv)
    # 4
    y_sa = linear(attention(q, k, v, H, dh), w["w_o"], w["b_o"])
    xr = x[sel] + g1 * y_sa
    # 5: cross-attention with TGAA
    hc = layernorm(xr) * np.asarray(w["ln3_w"], F64) + np.asarray(w["ln3_b"], F64)
    qc = rmsnorm(linear(hc, w["w_cq"], w["b_cq"]), w["g_cq"])
    ctx = np.asarray(text_ctx, F64)
    wck, wcv = np.asarray(w["w_ckv"], F64)[:D], np.asarray(w["w_ckv"], F64)[D:]
    bck, bcv = np.asarray(w["b_ckv"], F64)[:D], np.asarray(w["b_ckv"], F64)[D:]
    kc = rmsnorm(linear(ctx, wck, bck), w["g_ck"])
    vc = linear(ctx, wcv, bcv)
    kc_amp = tgaa_amplify_keys(kc, key_scale)
    y_ca = linear(attention(qc, kc_amp, vc, H, dh), w["w_co"], w["b_co"])
    xr = xr + gamma_o * y_ca
    # 6: FFN
    h2 = layernorm(xr) * (1.0 + sc2) + sh2
    y_ffn = linear(gelu_tanh(linear(h2, w["w_1"], w["b_1"])), w["w_2"], w["b_2"])
    out = xr + g2 * y_ffn
    if return_branches:
        return out, dict(y_sa=y_sa, y_ca=y_ca, y_ffn=y_ffn, g1=g1, g2=g2)
    return out


# --------------------------------------------------------------------------
# Region masks (Sec. 3.3.1 "Region Mask Generation", stages 2-3; Sec. 3.3.2, Eq. 5)
# --------------------------------------------------------------------------

def mask_propagate_keyframes(key_masks, frame_key):
    """Key-frame strategy of the pixel-space segmentation stage: masks exist only for
    the key frames; frame f takes the mask of the key frame of its temporal group,
    frame_key[f]. key_masks [Kf, Hp, Wp] -> [Tp, Hp, Wp]. How frames are grouped is
    not fixed by the paper, so the assignment is an input."""
    km = np.asarray(key_masks) != 0
    fk = np.asarray(frame_key, np.int64)
    assert fk.ndim == 1 and (fk >= 0).all() and (fk < km.shape[0]).all()
    return km[fk].astype(np.uint8)


def pooled_extent(n, k, lead=0):
    """Number of windows along one axis: `lead` leading sites are windows of their own
    (a causal video VAE encodes the first frame alone), the rest is cut into windows of
    k, the last one possibly short."""
    assert k >= 1 and 0 <= lead <= n
    return lead + -(-(n - lead) // k)


def mask_maxpool(mask, window, t_lead=0):
    """Latent-space projection: the binary mask is downsampled with a max pool
    (stride = window, windows that run over the edge are cut at the edge).
    mask [Tp, Hp, Wp], window (kt, kh, kw). Along time the first t_lead frames map
    to one output frame each. A window is set iff any site in it is set."""
    m = np.asarray(mask) != 0
    Tp, Hp, Wp = m.shape
    kt, kh, kw = window
    To, Ho, Wo = pooled_extent(Tp, kt, t_lead), pooled_extent(Hp, kh), pooled_extent(Wp, kw)
    out = np.zeros((To, Ho, Wo), np.uint8)
    for t in range(To):
        if t < t_lead:
            t0, t1 = t, t + 1
        else:
            t0 = t_lead + (t - t_lead) * kt
            t1 = min(t0 + kt, Tp)
        for y in range(Ho):
            rows = m[t0:t1, y * kh:min((y + 1) * kh, Hp), :]
            col_any = rows.any(axis=(0, 1))                       # [Wp]
            for x in range(Wo):
                out[t, y, x] = col_any[x * kw:min((x + 1) * kw, Wp)].any()
    return out


def mask_dilate(mask_base, radius):
    """Eq. 5: I(M_base * K_r > 0) with K_r the all-ones kernel of (2 r_a + 1) sites
    along each axis a. The convolution is written out as a sum of shifted copies of
    the zero-padded mask (sites beyond the grid count as 0). The paper gives one
    radius r; a radius per axis (rt, rh, rw) covers both a purely spatial kernel
    (rt = 0) and a spatio-temporal one."""
    m = (np.asarray(mask_base) != 0).astype(np.int64)
    assert m.ndim == 3
    rt, rh, rw = radius
    assert rt >= 0 and rh >= 0 and rw >= 0
    T, H, W = m.shape
    padded = np.pad(m, ((rt, rt), (rh, rh), (rw, rw)))
    conv = np.zeros_like(m)
    for dt in range(2 * rt + 1):
        for dy in range(2 * rh + 1):
            for dx in range(2 * rw + 1):
                conv += padded[dt:dt + T, dy:dy + H, dx:dx + W]
    return (conv > 0).astype(np.uint8)


def mask_hierarchy(mask_base, r_edit, r_see):
    """Eq. 5: (M_edit, M_see) from M_base with r_see >= r_edit on every axis, which
    gives M_see >= M_edit >= M_base site by site."""
    assert all(a >= b for a, b in zip(r_see, r_edit))
    return mask_dilate(mask_base, r_edit), mask_dilate(mask_base, r_see)


# --------------------------------------------------------------------------
# Selective region path (Sec. 3.3; Eq. 6)
# --------------------------------------------------------------------------


def region_compact(mask_see):
    """Ascending token ids where the visible mask is set."""
    return np.flatnonzero(np.asarray(mask_see) != 0).astype(np.int64)


def gather_rows(x, idx):
    return np.asarray(x)[np.asarray(idx, np.int64)].copy()


def scatter_rows(dst, src, idx):
    out = np.array(dst, copy=True)
    out[np.asarray(idx, np.int64)] = src
    return out


def expand_token_mask(mask_tok, grid, patch, C):
    """Token-grid mask [T*Hg*Wg] -> latent-shaped [C, T*pt, Hg*ph, Wg*pw]."""
    T, Hg, Wg = grid
    pt, ph, pw = patch
    m = np.asarray(mask_tok).reshape(T, Hg, Wg)
    m = np.repeat(np.repeat(np.repeat(m, pt, 0), ph, 1), pw, 2)
    return np.broadcast_to(m[None], (C,) + m.shape)


def region_blend(L, SL, mask_edit_tok, grid, patch):
    """Eq. 6: L <- M_edit * L + (1 - M_edit) * SL, M_edit binary, given per token."""
    L = np.asarray(L)
    SL = np.asarray(SL)
    M = (expand_token_mask(mask_edit_tok, grid, patch, L.shape[0]) != 0).astype(L.dtype)
    return M * L + (1 - M) * SL


# --------------------------------------------------------------------------
# Step glue: declared stand-ins that close the denoising loop around the blocks
# (the paper's sampler is DPM++ with default settings, Sec. 4.1; the Euler flow-matching update
#  used here is that solver's first-order step, the multistep form follows further down)
# --------------------------------------------------------------------------


def patchify(latent, patch):
    """[C, T, Hl, Wl] -> [L, C*pt*ph*pw]; token order (t, hg, wg), feature order (c, dt, dy, dx)."""
    C, T, Hl, Wl = latent.shape
    pt, ph, pw = patch
    z = np.asarray(latent).reshape(C, T // pt, pt, Hl // ph, ph, Wl // pw, pw)
    return z.transpose(1, 3, 5, 0, 2, 4, 6).reshape((T // pt) * (Hl // ph) * (Wl // pw), C * pt * ph * pw)


def unpatchify(tokens, latent_shape, patch):
    C, T, Hl, Wl = latent_shape
    pt, ph, pw = patch
    z = np.asarray(tokens).reshape(T // pt, Hl // ph, Wl // pw, C, pt, ph, pw)
    return z.transpose(3, 0, 4, 1, 5, 2, 6).reshape(C, T, Hl, Wl)


def text_project(text_emb, gw):
    """Raw text embeddings [Lt, text_dim] -> context [Lt, D]: linear, tanh-GELU, linear."""
    return linear(gelu_tanh(linear(text_emb, gw["w_text1"], gw["b_text1"])), gw["w_text2"], gw["b_text2"])


def sinusoidal_features(t, freq_dim):
    """[cos(t w_i), sin(t w_i)] with w_i = 10000^(-i / half), i < half = freq_dim / 2."""
    half = freq_dim // 2
    w = np.power(10000.0, -np.arange(half, dtype=F64) / half)
    a = float(t) * w
    return np.concatenate([np.cos(a), np.sin(a)])


def silu(x):
    x = np.asarray(x, F64)
    return x / (1.0 + np.exp(-x))


def time_mod(t, tw, D, freq_dim=256):
    """Timestep injection (Sec. 2.1 / Fig. 2 name it; the arithmetic is the Wan2.1-shaped one):
    e = W2 silu(W1 f(t) + b1) + b2 with f the sinusoidal features; the six modulation rows of every
    block are t_mod = reshape(Wp silu(e) + bp, [6, D]); the head takes e itself in both of its rows."""
    f = sinusoidal_features(t, freq_dim)
    e = linear(silu(linear(f, tw["w_t1"], tw["b_t1"])), tw["w_t2"], tw["b_t2"])
    t_mod = linear(silu(e), tw["w_tp"], tw["b_tp"]).reshape(6, D)
    t_head = np.stack([e, e])
    return t_mod, t_head


def patch_embed(patches, gw):
    return linear(patches, gw["w_patch"], gw["b_patch"])


def head(x, gw, t_head):
    """Output head: LN(x)(1 + scale) + shift with (shift, scale) = head_table + t_head, then linear to a patch."""
    sh, sc = np.asarray(gw["head_table"], F64) + np.asarray(t_head, F64)
    return linear(layernorm(x) * (1.0 + sc) + sh, gw["w_head"], gw["b_head"])


def denoise_step(latent, blocks, gw, shape, text_ctx, t_mod, t_head, dsigma,
                 mask_see=None, mask_edit=None, SL=None, key_scale=None, gamma_o=1.0):
    """One computed denoising step (stage 2 when masks are given, else stage 3).

    Stage 2 (Sec. 3.3): the tokens in M_see are compacted, run through every block
    (self-attention over exactly those tokens), the sampler updates only them, and
    Eq. 6 merges the result with the source latent SL under M_edit.
    """
    lat = np.asarray(latent, F64)
    patch = shape.patch
    Ltok = shape.L
    idx = np.arange(Ltok) if mask_see is None else region_compact(mask_see)
    toks = patchify(lat, patch)
    x = patch_embed(gather_rows(toks, idx), gw)
    for w in blocks:
        x = dit_block(x, w, shape, text_ctx, t_mod, token_idx=idx, key_scale=key_scale, gamma_o=gamma_o)
    v = head(x, gw, t_head)
    toks_new = scatter_rows(toks, gather_rows(toks, idx) + dsigma * v, idx)
    out = unpatchify(toks_new, lat.shape, patch)
    if mask_edit is not None:
        out = region_blend(out, np.asarray(SL, F64), mask_edit, shape.grid, patch)
    return out


def run_schedule(plan, sigmas, latent0, SL, blocks, gw, shape, text_ctx, t_mods, t_heads,
                 mask_see=None, mask_edit=None, key_scale_of=None, store_after=None):
    """The three-stage loop (Sec. 3.1): stage-1 steps take the source latent as is,
    stage-2 steps run the selective region path, stage-3 steps run everything.
    key_scale_of(gamma_k) builds the per-text-token key scale for a step.
    With store_after = k the latent after k steps (the intermediate state a cache update keeps)
    is returned as well; with a list of depths, the list of those states."""
    lat = np.asarray(latent0, F64)
    if store_after is not None and not np.isscalar(store_after):
        depths = [int(k) for k in store_after]
        snaps = {}
        for k in sorted(set(depths)):
            assert 1 <= k <= len(plan)
            snaps[k] = run_schedule(plan[:k], sigmas, lat, SL, blocks, gw, shape, text_ctx, t_mods, t_heads,
                                    mask_see=mask_see, mask_edit=mask_edit, key_scale_of=key_scale_of)
        final = run_schedule(plan, sigmas, lat, SL, blocks, gw, shape, text_ctx, t_mods, t_heads,
                             mask_see=mask_see, mask_edit=mask_edit, key_scale_of=key_scale_of)
        return final, [snaps[k] for k in depths]
    snap = None
    for i, (stage, gk, go) in enumerate(plan):
        if store_after is not None and i == store_after:
            snap = lat.copy()
        if stage == 1:
            lat = np.asarray(SL, F64).copy()
            continue
        ks = key_scale_of(gk) if key_scale_of is not None else None
        ds = sigmas[i + 1] - sigmas[i]
        if stage == 2:
            lat = denoise_step(lat, blocks, gw, shape, text_ctx, t_mods[i], t_heads[i], ds,
                               mask_see=mask_see, mask_edit=mask_edit, SL=SL, key_scale=ks, gamma_o=go)
        else:
            lat = denoise_step(lat, blocks, gw, shape, text_ctx, t_mods[i], t_heads[i], ds,
                               key_scale=ks, gamma_o=go)
    if store_after is not None:
        return lat, (lat.copy() if store_after == len(plan) else snap)
    return lat


# --------------------------------------------------------------------------
# Sampler (Sec. 4.1 names the DPM++ solver with default settings and gives no formulas):
# DPM-Solver++ in data-prediction form, multistep, order <= 2, as published by its authors,
# on the rectified-flow path x_sigma = alpha x0 + sigma eps with alpha = 1 - sigma, the path
# the Wan2.1 models are trained on. Notation of the solver paper: lambda = log(alpha / sigma),
# h = lambda_t - lambda_s, r = h_prev / h, D = the (extrapolated) data prediction.
# --------------------------------------------------------------------------


def flow_alpha(sigma):
    return 1.0 - np.asarray(sigma, F64)


def flow_lambda(sigma):
    """Half log-SNR of the rectified-flow path; +inf at sigma = 0, -inf at sigma = 1."""
    sigma = np.asarray(sigma, F64)
    with np.errstate(divide="ignore"):
        return np.log(flow_alpha(sigma)) - np.log(sigma)


def velocity_to_x0(x, v, sigma):
    """The models predict the velocity v = eps - x0 of the path, so x0 = x - sigma v."""
    return np.asarray(x, F64) - float(sigma) * np.asarray(v, F64)


def cfg_combine(v_cond, v_uncond, guidance):
    """Classifier-free guidance: v = v_uncond + g (v_cond - v_uncond)."""
    v_cond = np.asarray(v_cond, F64)
    v_uncond = np.asarray(v_uncond, F64)
    return v_uncond + float(guidance) * (v_cond - v_uncond)


def dpmpp_update(x_s, D, sigma_s, sigma_t):
    """x_t = (sigma_t / sigma_s) x_s - alpha_t (exp(-h) - 1) D: the exact solution of the
    diffusion ODE from s to t when the data prediction is the constant D."""
    with np.errstate(invalid="ignore"):
        h = flow_lambda(sigma_t) - flow_lambda(sigma_s)
    h = np.inf if np.isnan(h) else h          # sigma_s = 1 and sigma_t = 0 at once: one step over the whole path
    return (sigma_t / sigma_s) * np.asarray(x_s, F64) - flow_alpha(sigma_t) * np.expm1(-h) * np.asarray(D, F64)


def dpmpp_first_order(x_s, x0_s, sigma_s, sigma_t):
    return dpmpp_update(x_s, x0_s, sigma_s, sigma_t)


def dpmpp_2m(x_s, x0_s, x0_prev, sigma_prev, sigma_s, sigma_t):
    """Second-order multistep update: D = x0_s + (x0_s - x0_prev) / (2 r), r = h_prev / h, the
    linear extrapolation in lambda of the last two data predictions to the middle of the step."""
    lam_prev, lam_s, lam_t = flow_lambda(sigma_prev), flow_lambda(sigma_s), flow_lambda(sigma_t)
    h = lam_t - lam_s
    h_prev = lam_s - lam_prev
    r = h_prev / h
    x0_s = np.asarray(x0_s, F64)
    D = x0_s + (x0_s - np.asarray(x0_prev, F64)) / (2.0 * r)
    return dpmpp_update(x_s, D, sigma_s, sigma_t)


def model_velocity(latent, idx, blocks, gw, shape, text_ctx, t_mod, t_head, key_scale=None, gamma_o=1.0):
    """The model's velocity prediction on the tokens idx: patch embedding, every block, head."""
    toks = patchify(np.asarray(latent, F64), shape.patch)
    x = patch_embed(gather_rows(toks, idx), gw)
    for w in blocks:
        x = dit_block(x, w, shape, text_ctx, t_mod, token_idx=idx, key_scale=key_scale, gamma_o=gamma_o)
    return head(x, gw, t_head)


def denoise_step_dpmpp(latent, blocks, gw, shape, text_ctx, t_mod, t_head, sigma_prev, sigma_s, sigma_t,
                       x0_prev, hist, order=2, text_ctx_uncond=None, guidance=1.0,
                       mask_see=None, mask_edit=None, SL=None, key_scale=None, gamma_o=1.0):
    """One computed step with the DPM-Solver++ update in place of the Euler one.

    x0_prev is latent-shaped and holds the previous step's data prediction where hist (one
    flag per token) is set. A token takes the second-order update when order >= 2, it has
    history, and the step does not end at sigma = 0 (there h is infinite and only the
    first-order form is defined); otherwise the first-order one. With text_ctx_uncond the model
    runs twice and the velocities are combined by classifier-free guidance; TGAA belongs to the
    conditional branch only (an unconditional prompt has no differential tokens).
    Returns (latent, x0 history, history flags) after the step.
    """
    lat = np.asarray(latent, F64)
    patch = shape.patch
    idx = np.arange(shape.L) if mask_see is None else region_compact(mask_see)
    v = model_velocity(lat, idx, blocks, gw, shape, text_ctx, t_mod, t_head, key_scale=key_scale, gamma_o=gamma_o)
    if text_ctx_uncond is not None:
        v_u = model_velocity(lat, idx, blocks, gw, shape, text_ctx_uncond, t_mod, t_head)
        v = cfg_combine(v, v_u, guidance)
    toks = patchify(lat, patch)
    x_s = gather_rows(toks, idx)
    x0 = velocity_to_x0(x_s, v, sigma_s)
    new = dpmpp_first_order(x_s, x0, sigma_s, sigma_t)
    use = np.asarray(hist).reshape(-1)[idx] != 0
    if order >= 2 and sigma_t > 0.0 and use.any():
        x0_old = gather_rows(patchify(np.asarray(x0_prev, F64), patch), idx)
        second = dpmpp_2m(x_s, x0, x0_old, sigma_prev, sigma_s, sigma_t)
        new = np.where(use[:, None], second, new)
    out = unpatchify(scatter_rows(toks, new, idx), lat.shape, patch)
    if mask_edit is not None:
        out = region_blend(out, np.asarray(SL, F64), mask_edit, shape.grid, patch)
    x0_hist = unpatchify(scatter_rows(patchify(np.asarray(x0_prev, F64), patch), x0, idx), lat.shape, patch)
    hist_new = np.zeros(shape.L, np.uint8)
    hist_new[idx] = 1
    return out, x0_hist, hist_new


def run_schedule_dpmpp(plan, sigmas, latent0, SL, blocks, gw, shape, text_ctx, t_mods, t_heads, order=2,
                       text_ctx_uncond=None, guidance=1.0, mask_see=None, mask_edit=None, key_scale_of=None):
    """The three-stage loop with the multistep solver. History starts empty at the first
    computed step; a token skipped by a step (outside M_see in stage 2) has none in the next."""
    lat = np.asarray(latent0, F64)
    x0_prev = np.zeros_like(lat)
    hist = np.zeros(shape.L, np.uint8)
    for i, (stage, gk, go) in enumerate(plan):
        if stage == 1:
            lat = np.asarray(SL, F64).copy()
            continue
        ks = key_scale_of(gk) if key_scale_of is not None else None
        s_prev = sigmas[i - 1] if i > 0 else sigmas[i]
        kw = dict(order=order, text_ctx_uncond=text_ctx_uncond, guidance=guidance, key_scale=ks, gamma_o=go)
        if stage == 2:
            kw.update(mask_see=mask_see, mask_edit=mask_edit, SL=SL)
        lat, x0_prev, hist = denoise_step_dpmpp(lat, blocks, gw, shape, text_ctx, t_mods[i], t_heads[i], s_prev,
                                                sigmas[i], sigmas[i + 1], x0_prev, hist, **kw)
    return lat
