"""Seeded synthetic inputs for the Chorus hot path.

This module only draws numbers and lays them out. It holds none of the method's
arithmetic (no attention, no normalisation of activations, no schedule): both the
CPU oracle's tests and the HIP path's tests/bench take their inputs from here so
that the two sides see identical bits.

Every tensor gets its own Philox stream keyed by (master seed, tensor name), so
adding or reordering tensors never changes the values of another tensor.

Shapes follow the configurations the benchmark is quoted on: a Wan2.1-shaped DiT
block (hidden D, H heads of dh, FFN width F, Lt text tokens), a latent
[C, T, Hl, Wl] patchified 1x2x2 into a token grid (T, Hl/2, Wl/2), and a prompt
embedding cache [N, d] of unit-norm rows.
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass, field

import numpy as np

__all__ = [
    "stream", "normal", "to_bf16_bits", "bf16_bits_to_f32", "round_bf16",
    "BlockShape", "SHAPES", "block_weights", "block_inputs", "stress_block_weights",
    "cache_embeddings", "cache_query", "box_mask", "bernoulli_mask", "exact_count_mask",
    "tdiff_scale", "latent", "glue_weights",
]


def stream(seed: int, name: str) -> np.random.Generator:
    """Philox generator keyed by (seed, name)."""
    h = hashlib.sha256(f"{seed}:{name}".encode()).digest()
    key = int.from_bytes(h[:16], "little")
    return np.random.Generator(np.random.Philox(key=key))


def normal(seed: int, name: str, shape, std: float = 1.0, mean: float = 0.0) -> np.ndarray:
    g = stream(seed, name)
    return (g.standard_normal(size=shape, dtype=np.float32) * np.float32(std) + np.float32(mean)).astype(np.float32)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit pattern (uint16), round to nearest even. Finite inputs only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 values rounded once to the nearest bf16-representable fp32."""
    return bf16_bits_to_f32(to_bf16_bits(x)).reshape(np.shape(x))


@dataclass(frozen=True)
class BlockShape:
    name: str
    D: int          # hidden width
    H: int          # heads
    dh: int         # head dim
    F: int          # FFN width
    Lt: int         # text tokens
    text_dim: int   # raw text embedding width (before projection to D)
    grid: tuple     # token grid (T, Hg, Wg)
    C: int = 16     # latent channels
    patch: tuple = (1, 2, 2)
    blocks: int = 1
    cache_N: int = 8
    cache_d: int = 256
    latent_std: float = 1.0
    text_std: float = 1.0

    @property
    def L(self) -> int:
        return self.grid[0] * self.grid[1] * self.grid[2]

    @property
    def latent_shape(self) -> tuple:
        return (self.C, self.grid[0] * self.patch[0], self.grid[1] * self.patch[1], self.grid[2] * self.patch[2])

    @property
    def patch_dim(self) -> int:
        return self.C * self.patch[0] * self.patch[1] * self.patch[2]


SHAPES = {
    # tiny single block: 4 frames x 8x8 patches
    "c1": BlockShape("c1", D=256, H=4, dh=64, F=1024, Lt=16, text_dim=256, grid=(4, 8, 8),
                     blocks=1, cache_N=8, cache_d=256, latent_std=0.02, text_std=0.02),
    # Wan2.1-1.3B-shaped 480p: latent 16x21x60x104
    "wan1p3b_480p": BlockShape("wan1p3b_480p", D=1536, H=12, dh=128, F=8960, Lt=512, text_dim=4096,
                               grid=(21, 30, 52), blocks=30, cache_N=4096, cache_d=4096),
    # reduced grid with the 1.3B widths, for whole-schedule oracle runs
    "wan1p3b_small": BlockShape("wan1p3b_small", D=1536, H=12, dh=128, F=8960, Lt=512, text_dim=4096,
                                grid=(5, 12, 20), blocks=2, cache_N=64, cache_d=4096),
    # the 1.3B widths on a grid of 2304 tokens: the smallest whole number of 256-row tiles that reaches the 2048 rows
    # from which the block runs its long-sequence self-attention kernel; still small enough for the full oracle
    "wan1p3b_mid": BlockShape("wan1p3b_mid", D=1536, H=12, dh=128, F=8960, Lt=512, text_dim=4096,
                              grid=(6, 16, 24), blocks=2, cache_N=64, cache_d=4096),
    # Wan2.1-14B-shaped 720p: latent 16x21x90x160
    "wan14b_720p": BlockShape("wan14b_720p", D=5120, H=40, dh=128, F=13824, Lt=512, text_dim=4096,
                              grid=(21, 45, 80), blocks=40, cache_N=4096, cache_d=4096),
}


def block_weights(shape: BlockShape, seed: int = 0, block: int = 0, std: float = 0.02) -> dict:
    """Random-init weights of one DiT block.

    Matrices are [out_features, in_features] and hold bf16-representable fp32
    values (the device stores them as bf16; the oracle reads the same values).
    Biases are zero, norm gains one, the modulation table ~N(0, std).
    """
    D, F = shape.D, shape.F
    p = f"block{block}."
    w = {}

    def mat(name, o, i):
        w[name] = round_bf16(normal(seed, p + name, (o, i), std))

    mat("w_qkv", 3 * D, D)
    mat("w_o", D, D)
    mat("w_cq", D, D)
    mat("w_ckv", 2 * D, D)
    mat("w_co", D, D)
    mat("w_1", F, D)
    mat("w_2", D, F)
    w["b_qkv"] = np.zeros(3 * D, np.float32)
    w["b_o"] = np.zeros(D, np.float32)
    w["b_cq"] = np.zeros(D, np.float32)
    w["b_ckv"] = np.zeros(2 * D, np.float32)
    w["b_co"] = np.zeros(D, np.float32)
    w["b_1"] = np.zeros(F, np.float32)
    w["b_2"] = np.zeros(D, np.float32)
    for g in ("g_q", "g_k", "g_cq", "g_ck", "ln3_w"):
        w[g] = np.ones(D, np.float32)
    w["ln3_b"] = np.zeros(D, np.float32)
    w["mod_table"] = normal(seed, p + "mod_table", (6, D), std)
    return w


def stress_block_weights(shape: BlockShape, seed: int = 0, block: int = 0) -> dict:
    """Variant that makes every branch matter: non-zero biases, q/k gains of 2
    (attention logits with std ~4, i.e. peaked rows), gates ~N(1, 0.1), non-trivial
    norm affine."""
    w = block_weights(shape, seed, block)
    D, F = shape.D, shape.F
    p = f"stress{block}."
    for b, n in (("b_qkv", 3 * D), ("b_o", D), ("b_cq", D), ("b_ckv", 2 * D), ("b_co", D), ("b_1", F), ("b_2", D)):
        w[b] = normal(seed, p + b, (n,), 0.05)
    for g in ("g_q", "g_k", "g_cq", "g_ck"):
        w[g] = normal(seed, p + g, (D,), 0.1, 2.0)
    w["ln3_w"] = normal(seed, p + "ln3_w", (D,), 0.1, 1.0)
    w["ln3_b"] = normal(seed, p + "ln3_b", (D,), 0.1)
    mt = normal(seed, p + "mod_table", (6, D), 0.1)
    mt[2] += 1.0  # self-attention gate
    mt[5] += 1.0  # FFN gate
    w["mod_table"] = mt
    return w


def block_inputs(shape: BlockShape, seed: int = 0, L: int | None = None, x_std: float | None = None) -> dict:
    """Hidden states x [L, D] fp32, projected text context [Lt, D] (bf16-representable),
    projected timestep modulation t_mod [6, D] fp32."""
    L = shape.L if L is None else L
    xs = shape.latent_std if x_std is None else x_std
    return {
        "x": normal(seed, "x", (L, shape.D), xs),
        "text_ctx": round_bf16(normal(seed, "text_ctx", (shape.Lt, shape.D), shape.text_std)),
        "t_mod": normal(seed, "t_mod", (6, shape.D), 0.02),
    }


def glue_weights(shape: BlockShape, seed: int = 0, std: float = 0.02) -> dict:
    """Weights around the block stack: patch embedding, text projection (two layers),
    output head with its own 2-row modulation table."""
    D, P = shape.D, shape.patch_dim
    w = {
        "w_patch": round_bf16(normal(seed, "glue.w_patch", (D, P), std)),
        "b_patch": np.zeros(D, np.float32),
        "w_text1": round_bf16(normal(seed, "glue.w_text1", (D, shape.text_dim), std)),
        "b_text1": np.zeros(D, np.float32),
        "w_text2": round_bf16(normal(seed, "glue.w_text2", (D, D), std)),
        "b_text2": np.zeros(D, np.float32),
        "w_head": round_bf16(normal(seed, "glue.w_head", (P, D), std)),
        "b_head": np.zeros(P, np.float32),
        "head_table": normal(seed, "glue.head_table", (2, D), std),
    }
    return w


def time_weights(shape: BlockShape, seed: int = 0, freq_dim: int = 256, std: float = 0.02) -> dict:
    """Weights of the timestep embedding: two layers on the sinusoidal features, then the projection to the six
    modulation rows of a block. Biases are non-zero so that every term matters."""
    D = shape.D
    return {
        "w_t1": round_bf16(normal(seed, "time.w_t1", (D, freq_dim), std)),
        "b_t1": normal(seed, "time.b_t1", (D,), std),
        "w_t2": round_bf16(normal(seed, "time.w_t2", (D, D), std)),
        "b_t2": normal(seed, "time.b_t2", (D,), std),
        "w_tp": round_bf16(normal(seed, "time.w_tp", (6 * D, D), std)),
        "b_tp": normal(seed, "time.b_tp", (6 * D,), std),
    }


def latent(shape: BlockShape, seed: int = 0, name: str = "latent", std: float | None = None) -> np.ndarray:
    return normal(seed, name, shape.latent_shape, shape.latent_std if std is None else std)


def _unit_rows(a: np.ndarray) -> np.ndarray:
    a64 = a.astype(np.float64)
    a64 /= np.linalg.norm(a64, axis=-1, keepdims=True)
    return a64.astype(np.float32)


def cache_embeddings(N: int, d: int, seed: int = 0, centroids: int = 256, spread: float = 0.5) -> np.ndarray:
    """Clustered unit-norm prompt embeddings: entry = unit(centroid + spread * n),
    n ~ N(0, I/d). Stand-in for one k-means cluster structure of real prompt embeddings."""
    c = _unit_rows(normal(seed, "cache.centroids", (min(centroids, max(N, 1)), d)))
    if N == 0:
        return np.zeros((0, d), np.float32)
    which = stream(seed, "cache.assign").integers(0, c.shape[0], size=N)
    noise = normal(seed, "cache.noise", (N, d), spread / np.sqrt(d))
    return _unit_rows(c[which] + noise)


def cache_query(cache: np.ndarray, seed: int = 0, near: int | None = None, spread: float = 0.5, trial: int = 0) -> np.ndarray:
    """A query: noisy copy of cache row `near` (a likely hit), or uniform on the sphere (a miss)."""
    d = cache.shape[1]
    if near is None:
        return _unit_rows(normal(seed, f"query.miss{trial}", (d,)))
    n = normal(seed, f"query.near{trial}", (d,), spread / np.sqrt(d))
    return _unit_rows(cache[near] + n)


def box_mask(grid, t: int, h: int, w: int, t0: int = 0, h0: int = 0, w0: int = 0) -> np.ndarray:
    """Contiguous spatio-temporal box on the token grid, uint8 [T*Hg*Wg]."""
    T, Hg, Wg = grid
    m = np.zeros((T, Hg, Wg), np.uint8)
    m[t0:t0 + t, h0:h0 + h, w0:w0 + w] = 1
    return m.reshape(-1)


def bernoulli_mask(L: int, p: float, seed: int = 0) -> np.ndarray:
    return (stream(seed, f"mask.bernoulli{p}").random(L) < p).astype(np.uint8)


def exact_count_mask(L: int, count: int, seed: int = 0) -> np.ndarray:
    m = np.zeros(L, np.uint8)
    m[stream(seed, "mask.exact").permutation(L)[:count]] = 1
    return m


def tdiff_scale(Lt: int, gamma_k: float, seed: int = 0, n_diff: int | None = None) -> np.ndarray:
    """Per-text-token key scale g_j: gamma_k on the differential tokens, 1 elsewhere.
    n_diff=None marks every token as differential."""
    g = np.ones(Lt, np.float32)
    if n_diff is None:
        g[:] = gamma_k
    else:
        g[stream(seed, "tdiff").permutation(Lt)[:n_diff]] = gamma_k
    return g


def pixel_key_masks(Kf: int, Hp: int, Wp: int, seed: int = 0, n_obj: int = 2, fill: float = 0.12) -> np.ndarray:
    """Stand-in for a segmentation model's output on the key frames: uint8 [Kf, Hp, Wp]
    with n_obj filled ellipses that drift and breathe from key frame to key frame, plus a
    few isolated pixels (segmentation speckle). `fill` is roughly the covered fraction."""
    g = stream(seed, f"mask.pixel.{Kf}x{Hp}x{Wp}")
    yy, xx = np.mgrid[0:Hp, 0:Wp]
    out = np.zeros((Kf, Hp, Wp), np.uint8)
    area = fill * Hp * Wp / max(1, n_obj)
    for _ in range(n_obj):
        cy, cx = g.uniform(0.2, 0.8) * Hp, g.uniform(0.2, 0.8) * Wp
        vy, vx = g.uniform(-0.02, 0.02) * Hp, g.uniform(-0.02, 0.02) * Wp
        aspect = g.uniform(0.6, 1.6)
        ry, rx = np.sqrt(area / np.pi * aspect), np.sqrt(area / np.pi / aspect)
        for k in range(Kf):
            s = 1.0 + 0.1 * np.sin(0.7 * k)
            e = ((yy - (cy + vy * k)) / (ry * s)) ** 2 + ((xx - (cx + vx * k)) / (rx * s)) ** 2 <= 1.0
            out[k] |= e.astype(np.uint8)
    n_speck = max(1, Hp * Wp // 50000)
    for k in range(Kf):
        out[k, g.integers(0, Hp, n_speck), g.integers(0, Wp, n_speck)] = 1
    return out


def frame_key_groups(Tp: int, Kf: int) -> np.ndarray:
    """Frame -> key-frame index for Kf contiguous temporal groups of (nearly) equal length."""
    return np.minimum(np.arange(Tp, dtype=np.int64) * Kf // max(1, Tp), Kf - 1).astype(np.int32)


def sparse_site_mask(shape3, count: int, seed: int = 0) -> np.ndarray:
    """uint8 [T, H, W] with exactly `count` isolated set sites (dilation / pooling edge cases)."""
    n = int(np.prod(shape3))
    m = np.zeros(n, np.uint8)
    m[stream(seed, f"mask.sparse.{shape3}").permutation(n)[:count]] = 1
    return m.reshape(shape3)
