"""ctypes binding of libchorus.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU (PyTorch is used
for device memory and streams, nothing else), checks dtype / contiguity, and
passes raw pointers, sizes and the current HIP stream through the C ABI declared
in include/chorus.h. Nothing here computes anything, and there is no fallback:
if the shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libchorus.so")
_lib = None

OK, E_ARG, E_SHAPE, E_WORKSPACE, E_HIP = 0, -1, -2, -3, -4
_ERR = {E_ARG: "CHORUS_E_ARG", E_SHAPE: "CHORUS_E_SHAPE", E_WORKSPACE: "CHORUS_E_WORKSPACE", E_HIP: "CHORUS_E_HIP"}


class ChorusError(RuntimeError):
    def __init__(self, fn, status, hip=0):
        self.status = status
        super().__init__(f"{fn} failed: {_ERR.get(status, status)}" + (f" (hipError {hip})" if status == E_HIP else ""))


class LookupResult(C.Structure):
    _fields_ = [("index", C.c_int32), ("score", C.c_float), ("hit", C.c_int32)]


class SchedParams(C.Structure):
    _fields_ = [("a1", C.c_double), ("b1", C.c_double), ("a2", C.c_double), ("b2", C.c_double), ("r3", C.c_int32),
                ("Gamma_k", C.c_double), ("Gamma_o", C.c_double), ("lam", C.c_double), ("gamma_override", C.c_double)]


class StepPlan(C.Structure):
    _fields_ = [("stage", C.c_int32), ("gamma_k", C.c_float), ("gamma_o", C.c_float)]


class BlockShape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("D", "H", "dh", "F", "Lt", "gT", "gH", "gW")]


_W_FIELDS = ["mod_table", "w_qkv", "b_qkv", "g_q", "g_k", "w_o", "b_o", "ln3_w", "ln3_b", "w_cq", "b_cq", "w_ckv",
             "b_ckv", "g_cq", "g_ck", "w_co", "b_co", "w_1", "b_1", "w_2", "b_2"]


class BlockWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _W_FIELDS]


class GlueWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("w_patch", "b_patch", "w_head", "b_head", "head_table")]


class ModelShape(C.Structure):
    _fields_ = [("block", BlockShape)] + [(n, C.c_int32) for n in ("C", "T", "Hl", "Wl", "ph", "pw", "n_blocks")]


class Request(C.Structure):
    _fields_ = [("cache_emb", C.c_void_p), ("cache_latents", C.c_void_p), ("cache_N", C.c_int64),
                ("cache_d", C.c_int32), ("query", C.c_void_p), ("tau", C.c_float),
                ("sched", C.POINTER(SchedParams)), ("n_steps", C.c_int32), ("sigmas", C.POINTER(C.c_float)),
                ("t_mods", C.c_void_p), ("t_heads", C.c_void_p), ("text_ctx", C.c_void_p), ("tdiff", C.c_void_p),
                ("mask_see", C.c_void_p), ("mask_edit", C.c_void_p), ("store_slot", C.c_int64),
                ("store_after", C.c_int32), ("latent_steps", C.POINTER(C.c_int32)), ("n_latent_steps", C.c_int32),
                ("solver_order", C.c_int32), ("text_ctx_uncond", C.c_void_p),
                ("guidance", C.c_float)]


class SamplerCoef(C.Structure):
    _fields_ = [(n, C.c_float) for n in ("sigma_s", "rho", "A", "c0", "c1")]


class TimeWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("w_t1", "b_t1", "w_t2", "b_t2", "w_tp", "b_tp")]


class RunResult(C.Structure):
    _fields_ = [("index", C.c_int32), ("score", C.c_float), ("hit", C.c_int32), ("K1", C.c_int32),
                ("K2", C.c_int32), ("Ls", C.c_int32)]


def lib_path() -> str:
    return _LIB_PATH


def load():
    """Loads the shared library (once). Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: run `python -m paper_2604_04451_amd.build` "
                          "(there is no CPU fallback for the HIP path)")
    lib = C.CDLL(_LIB_PATH)
    vp, i32, i64, f32, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_size_t
    sigs = {
        "chorus_version": (i32, []),
        "chorus_last_hip_error": (i32, []),
        "chorus_cache_lookup_workspace_bytes": (sz, [i64]),
        "chorus_cache_lookup": (i32, [vp, i64, i32, vp, f32, vp, vp, sz, vp]),
        "chorus_cache_lookup_static": (i32, [vp, i64, i32, vp, f32, vp, vp]),
        "chorus_cache_lowprec_bytes": (sz, [i64, i32, i32]),
        "chorus_cache_lowprec_store": (i32, [vp, i64, i32, i32, vp, vp]),
        "chorus_cache_lookup_lowprec_workspace_bytes": (sz, [i64]),
        "chorus_cache_lookup_lowprec": (i32, [vp, vp, i32, i64, i32, vp, f32, vp, vp, vp, sz, vp]),
        "chorus_cache_insert": (i32, [vp, vp, i64, i64, i32, i64, vp, vp, vp]),
        "chorus_cache_lookup_batch_workspace_bytes": (sz, [i64, i32, i32]),
        "chorus_cache_lookup_batch": (i32, [vp, i64, i32, vp, i32, f32, i32, vp, vp, vp, vp, sz, vp]),
        "chorus_denoise_schedule": (i32, [f32, f32, i32, C.POINTER(SchedParams), C.POINTER(i32), C.POINTER(i32),
                                          C.POINTER(StepPlan)]),
        "chorus_denoise_schedule_stored": (i32, [f32, f32, i32, C.POINTER(SchedParams), C.POINTER(i32), i32, C.POINTER(i32),
                                                 C.POINTER(i32), C.POINTER(i32), C.POINTER(StepPlan)]),
        "chorus_dit_block_workspace_bytes": (sz, [C.POINTER(BlockShape), i64]),
        "chorus_dit_block_step": (i32, [C.POINTER(BlockShape), C.POINTER(BlockWeights), vp, i64, vp, vp, vp, vp, f32,
                                        vp, sz, vp]),
        "chorus_text_kv_bytes": (sz, [C.POINTER(BlockShape)]),
        "chorus_text_kv_workspace_bytes": (sz, [C.POINTER(BlockShape)]),
        "chorus_text_kv_project": (i32, [C.POINTER(BlockShape), C.POINTER(BlockWeights), vp, vp, vp, sz, vp]),
        "chorus_dit_block_step_kv": (i32, [C.POINTER(BlockShape), C.POINTER(BlockWeights), vp, i64, vp, vp, vp, vp, f32,
                                           vp, sz, vp]),
        "chorus_region_blend": (i32, [vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp]),
        "chorus_region_compact_workspace_bytes": (sz, [i64]),
        "chorus_region_compact": (i32, [vp, i64, vp, vp, vp, sz, vp]),
        "chorus_region_gather_rows": (i32, [vp, vp, vp, i64, i64, vp]),
        "chorus_region_scatter_rows": (i32, [vp, vp, vp, i64, i64, vp]),
    }
    for name, (res, args) in sigs.items():
        fn = getattr(lib, name)  # AttributeError if the header and the library disagree
        fn.restype = res
        fn.argtypes = args
    lib._sigs = sigs
    _lib = lib
    _bind_ops(lib)
    return lib


def _bind_ops(lib):
    """Signatures of include/chorus_ops.h."""
    vp, i32, i64, f32, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_size_t
    GW, MS = C.POINTER(GlueWeights), C.POINTER(ModelShape)
    ops = {
        "chorus_gemm_bf16": (i32, [vp, vp, i64, i32, i32, i32, vp, vp, vp, vp, f32, vp]),
        "chorus_gemm_bf16_kernel": (i32, [vp, vp, i64, i32, i32, i32, vp, vp, vp, vp, f32, i32, vp]),
        "chorus_ln_modulate": (i32, [vp, vp, i64, i32, vp, vp, vp, vp, i32, vp]),
        "chorus_qk_norm_rope": (i32, [vp, i64, vp, vp, i64, i64, i32, i32, vp, i32, i32, i32, i32, f32, vp]),
        "chorus_v_transpose": (i32, [vp, i64, vp, i64, i64, i32, vp]),
        "chorus_attention": (i32, [vp, vp, vp, vp, vp, i64, i64, i64, i64, i32, i32, i32, vp]),
        "chorus_glue_workspace_bytes": (sz, [i32, i32, i64]),
        "chorus_patch_embed": (i32, [vp, i32, i32, i32, i32, i32, i32, vp, i64, GW, i32, vp, vp, sz, vp]),
        "chorus_head_update": (i32, [vp, vp, i64, vp, GW, vp, f32, i32, i32, i32, i32, i32, i32, i32, vp, sz, vp]),
        "chorus_head_update_region": (i32, [vp, vp, i64, vp, GW, vp, f32, vp, vp, i32, i32, i32, i32, i32, i32, i32, vp, sz,
                                            vp]),
        "chorus_text_project_workspace_bytes": (sz, [i32, i32]),
        "chorus_text_project": (i32, [vp, i32, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]),
        "chorus_denoise_step_workspace_bytes": (sz, [MS, i64]),
        "chorus_denoise_step": (i32, [MS, C.POINTER(BlockWeights), GW, vp, vp, i64, vp, vp, vp, vp, f32, f32, vp, vp,
                                      vp, sz, vp]),
        "chorus_denoise_run_workspace_bytes": (sz, [MS, i64]),
        "chorus_denoise_run": (i32, [MS, C.POINTER(BlockWeights), GW, C.POINTER(Request), vp, C.POINTER(RunResult), vp,
                                     sz, vp]),
        "chorus_stage1_copy": (i32, [vp, vp, i64, vp]),
        "chorus_model_text_kv_bytes": (sz, [MS]),
        "chorus_model_text_kv_project": (i32, [MS, C.POINTER(BlockWeights), vp, vp, vp, sz, vp]),
        "chorus_denoise_step_kv": (i32, [MS, C.POINTER(BlockWeights), GW, vp, vp, i64, vp, vp, vp, vp, f32, f32, vp, vp, vp,
                                         sz, vp]),
        "chorus_sampler_coefficients": (i32, [C.POINTER(f32), i32, i32, i32, C.POINTER(SamplerCoef)]),
        "chorus_head_solver_workspace_bytes": (sz, [i32, i32, i64, i32]),
        "chorus_head_update_solver": (i32, [vp, vp, vp, f32, i64, vp, GW, vp, C.POINTER(SamplerCoef), vp, vp, vp, vp, i32,
                                            i32, i32, i32, i32, i32, i32, vp, sz, vp]),
        "chorus_denoise_step_solver_workspace_bytes": (sz, [MS, i64, i32]),
        "chorus_denoise_step_solver": (i32, [MS, C.POINTER(BlockWeights), GW, vp, vp, i64, vp, vp, f32, vp, vp, vp, f32,
                                             C.POINTER(SamplerCoef), vp, vp, vp, vp, i32, vp, sz, vp]),
        "chorus_mask_pooled_extent": (i32, [i32, i32, i32]),
        "chorus_mask_project": (i32, [vp, i32, vp, i32, i32, i32, i32, i32, i32, i32, vp, vp]),
        "chorus_mask_hierarchy": (i32, [vp, i32, i32, i32, C.POINTER(i32), C.POINTER(i32), vp, vp, vp]),
        "chorus_time_mod_workspace_bytes": (sz, [i32, i32]),
        "chorus_time_mod": (i32, [f32, i32, i32, C.POINTER(TimeWeights), vp, vp, vp, sz, vp]),
        "chorus_mfma_ceiling_workspace_bytes": (sz, []),
        "chorus_mfma_ceiling": (i32, [i32, i32, i32, C.POINTER(C.c_double), vp, sz, vp]),
        "chorus_prof_enable": (i32, [i32]),
        "chorus_prof_reset": (i32, []),
        "chorus_prof_read": (i32, [i32, C.POINTER(C.c_double), C.POINTER(i32)]),
    }
    for name, (res, args) in ops.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    lib._sigs.update(ops)


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _p(t):
    return C.c_void_p(0 if t is None else t.data_ptr())


def _chk(t, dtype, name, shape=None):
    if t is None:
        return
    if not t.is_cuda:
        raise TypeError(f"{name}: device tensor required")
    if t.dtype != dtype:
        raise TypeError(f"{name}: expected {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise TypeError(f"{name}: must be contiguous")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise TypeError(f"{name}: expected shape {tuple(shape)}, got {tuple(t.shape)}")


def _status(fn, st):
    if st != OK:
        raise ChorusError(fn, st, load().chorus_last_hip_error())


def _ws(nbytes, device):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


# ---------------------------------------------------------------- lookup

def chorus_cache_lookup(cache_emb, query, tau, out=None, ws=None):
    """Returns a device int32 tensor [3] viewing (index, score bits, hit); use lookup_result() to read it."""
    lib = load()
    _chk(cache_emb, torch.float32, "cache_emb")
    _chk(query, torch.float32, "query")
    N, d = cache_emb.shape
    if query.numel() != d:
        raise TypeError("query: wrong length")
    if out is None:
        out = torch.empty(3, dtype=torch.int32, device=query.device)
    need = lib.chorus_cache_lookup_workspace_bytes(N)
    if ws is None:
        ws = _ws(need, query.device)
    _status("chorus_cache_lookup", lib.chorus_cache_lookup(_p(cache_emb) if N else C.c_void_p(0), N, d, _p(query),
                                                           float(tau), _p(out), _p(ws), ws.numel(), _stream()))
    return out


def chorus_cache_lookup_static(cache_emb, query, tau, out):
    """chorus_cache_lookup without a workspace (the library's own per-GPU scratch array); `out` is required so
    that this wrapper allocates nothing either."""
    lib = load()
    _chk(cache_emb, torch.float32, "cache_emb")
    _chk(query, torch.float32, "query")
    if out is None:
        raise TypeError("out: required")
    _chk(out, torch.int32, "out", (3,))
    N, d = cache_emb.shape
    if query.numel() != d:
        raise TypeError("query: wrong length")
    _status("chorus_cache_lookup_static", lib.chorus_cache_lookup_static(_p(cache_emb) if N else C.c_void_p(0), N, d,
                                                                         _p(query), float(tau), _p(out), _stream()))
    return out


LP_BF16, LP_FP8 = 0, 1


def chorus_cache_lowprec_store(emb, fmt, out=None):
    """Low-precision copy of fp32 rows [n, d]: a uint16 (bf16 bits) or uint8 (FP8 E4M3 codes) device tensor [n, d]."""
    lib = load()
    _chk(emb, torch.float32, "emb")
    n, d = emb.shape
    if out is None:
        out = torch.empty(n, d, dtype=torch.int16 if fmt == LP_BF16 else torch.uint8, device=emb.device)
    _status("chorus_cache_lowprec_store", lib.chorus_cache_lowprec_store(_p(emb) if n else C.c_void_p(0), n, d, int(fmt),
                                                                         _p(out) if n else C.c_void_p(0), _stream()))
    return out


def chorus_cache_lookup_lowprec(cache_emb, cache_lp, fmt, query, tau, out=None, n_rescored=None, ws=None):
    """Returns (result words [3] int32 as chorus_cache_lookup, n_rescored [1] int32), both on the device."""
    lib = load()
    _chk(cache_emb, torch.float32, "cache_emb")
    _chk(query, torch.float32, "query")
    N, d = cache_emb.shape
    if tuple(cache_lp.shape) != (N, d) or cache_lp.element_size() != (2 if fmt == LP_BF16 else 1) or not cache_lp.is_cuda:
        raise TypeError("cache_lp: wrong shape or element size")
    if query.numel() != d:
        raise TypeError("query: wrong length")
    if out is None:
        out = torch.empty(3, dtype=torch.int32, device=query.device)
    if n_rescored is None:
        n_rescored = torch.empty(1, dtype=torch.int32, device=query.device)
    if ws is None:
        ws = _ws(lib.chorus_cache_lookup_lowprec_workspace_bytes(N), query.device)
    _status("chorus_cache_lookup_lowprec",
            lib.chorus_cache_lookup_lowprec(_p(cache_emb) if N else C.c_void_p(0), _p(cache_lp) if N else C.c_void_p(0),
                                            int(fmt), N, d, _p(query), float(tau), _p(out), _p(n_rescored), _p(ws),
                                            ws.numel(), _stream()))
    return out, n_rescored


def chorus_cache_lookup_batch(cache_emb, queries, tau, k=1, ws=None):
    """Top-k entries for each row of queries: (index [Q, k] int32, score [Q, k] fp32, hit [Q] int32) on the device."""
    lib = load()
    _chk(cache_emb, torch.float32, "cache_emb")
    _chk(queries, torch.float32, "queries")
    N, d = cache_emb.shape
    Q = queries.shape[0]
    if queries.dim() != 2 or queries.shape[1] != d:
        raise TypeError("queries: expected [Q, d]")
    dev = queries.device
    idx = torch.empty(Q, k, dtype=torch.int32, device=dev)
    sc = torch.empty(Q, k, dtype=torch.float32, device=dev)
    hit = torch.empty(Q, dtype=torch.int32, device=dev)
    if ws is None:
        ws = _ws(lib.chorus_cache_lookup_batch_workspace_bytes(N, d, Q), dev)
    _status("chorus_cache_lookup_batch",
            lib.chorus_cache_lookup_batch(cache_emb.data_ptr() if N else 0, N, d, _p(queries), Q, float(tau), int(k), _p(idx),
                                          _p(sc), _p(hit), _p(ws), ws.numel(), _stream()))
    return idx, sc, hit


def lookup_result(out):
    """Host read-back of a lookup result tensor: (index, score, hit)."""
    h = out.cpu()
    return int(h[0]), float(h[1:2].view(torch.float32)[0]), bool(h[2])


# -------------------------------------------------------------- schedule

def chorus_denoise_schedule(m, tau, N, params=None, stored_steps=None):
    """(K1, K2, plan); with stored_steps (the depths the matched entry holds) also the position of the
    depth that full reuse resumes from, -1 if none: (K1, K2, plan, slot)."""
    lib = load()
    sp = None
    if params is not None:
        d = dict(a1=0.25, b1=0.25, a2=0.25, b2=0.25, r3=1, Gamma_k=1.5, Gamma_o=1.5, lam=0.5, gamma_override=0.0)
        d.update(params)
        sp = SchedParams(**d)
    plan = (StepPlan * max(N, 1))()
    k1, k2 = C.c_int32(0), C.c_int32(0)
    if stored_steps is not None:
        ss = (C.c_int32 * max(len(stored_steps), 1))(*[int(v) for v in stored_steps])
        slot = C.c_int32(0)
        _status("chorus_denoise_schedule_stored",
                lib.chorus_denoise_schedule_stored(float(m), float(tau), int(N), C.byref(sp) if sp is not None else None, ss,
                                                   len(stored_steps), C.byref(k1), C.byref(k2), C.byref(slot), plan))
        return k1.value, k2.value, [(plan[i].stage, plan[i].gamma_k, plan[i].gamma_o) for i in range(N)], slot.value
    _status("chorus_denoise_schedule",
            lib.chorus_denoise_schedule(float(m), float(tau), int(N), C.byref(sp) if sp is not None else None,
                                        C.byref(k1), C.byref(k2), plan))
    return k1.value, k2.value, [(plan[i].stage, plan[i].gamma_k, plan[i].gamma_o) for i in range(N)]


def chorus_cache_insert(cache_emb, cache_latents, slot, emb, latent):
    """Overwrites cache entry `slot` with the embedding and the latent (device copies)."""
    _chk(cache_emb, torch.float32, "cache_emb")
    _chk(cache_latents, torch.float32, "cache_latents")
    _chk(emb, torch.float32, "emb")
    _chk(latent, torch.float32, "latent")
    cap, d = cache_emb.shape
    elems = latent.numel()
    if emb.numel() != d or cache_latents.shape[0] != cap or cache_latents[0].numel() != elems:
        raise TypeError("cache_insert: shapes do not match")
    _status("chorus_cache_insert", load().chorus_cache_insert(_p(cache_emb), _p(cache_latents), cap, int(slot), d, elems,
                                                              _p(emb), _p(latent), _stream()))


# ---------------------------------------------------------------- region

def chorus_region_compact(mask, idx_out=None, count_out=None, ws=None):
    lib = load()
    _chk(mask, torch.uint8, "mask")
    L = mask.numel()
    if idx_out is None:
        idx_out = torch.empty(max(L, 1), dtype=torch.int32, device=mask.device)
    if count_out is None:
        count_out = torch.empty(1, dtype=torch.int32, device=mask.device)
    if ws is None:
        ws = _ws(lib.chorus_region_compact_workspace_bytes(L), mask.device)
    _status("chorus_region_compact",
            lib.chorus_region_compact(_p(mask), L, _p(idx_out), _p(count_out), _p(ws), ws.numel(), _stream()))
    return idx_out, count_out


def chorus_region_gather_rows(dst, src, idx, Ls=None):
    lib = load()
    _chk(idx, torch.int32, "idx")
    Ls = idx.numel() if Ls is None else Ls
    row_bytes = src.shape[-1] * src.element_size()
    assert dst.is_contiguous() and src.is_contiguous() and dst.dtype == src.dtype and dst.shape[-1] == src.shape[-1]
    assert dst.shape[0] >= Ls
    _status("chorus_region_gather_rows", lib.chorus_region_gather_rows(_p(dst), _p(src), _p(idx), Ls, row_bytes, _stream()))
    return dst


def chorus_region_scatter_rows(dst, src, idx, Ls=None):
    lib = load()
    _chk(idx, torch.int32, "idx")
    Ls = idx.numel() if Ls is None else Ls
    row_bytes = src.shape[-1] * src.element_size()
    assert dst.is_contiguous() and src.is_contiguous() and dst.dtype == src.dtype and dst.shape[-1] == src.shape[-1]
    assert src.shape[0] >= Ls
    _status("chorus_region_scatter_rows", lib.chorus_region_scatter_rows(_p(dst), _p(src), _p(idx), Ls, row_bytes, _stream()))
    return dst


def chorus_region_blend(out, L, SL, mask_edit, patch_hw=(2, 2)):
    lib = load()
    _chk(L, torch.float32, "L")
    _chk(SL, torch.float32, "SL", L.shape)
    _chk(out, torch.float32, "out", L.shape)
    _chk(mask_edit, torch.uint8, "mask_edit")
    Cc, T, H, W = L.shape
    ph, pw = patch_hw
    if mask_edit.numel() != T * (H // ph) * (W // pw):
        raise TypeError("mask_edit: wrong size")
    _status("chorus_region_blend", lib.chorus_region_blend(_p(out), _p(L), _p(SL), _p(mask_edit), Cc, T, H, W, ph, pw, _stream()))
    return out


# ----------------------------------------------------------------- block

@dataclass
class DeviceBlock:
    """Device copies of one block's weights plus the C struct that points at them."""
    tensors: dict
    cstruct: BlockWeights


def make_block_shape(D, H, dh, F, Lt, grid):
    return BlockShape(D, H, dh, F, Lt, grid[0], grid[1], grid[2])


def upload_block_weights(w: dict, device="cuda") -> DeviceBlock:
    """Copies numpy weights to the device: matrices as bf16 (values must already be
    bf16-representable), vectors and tables as fp32."""
    import numpy as np
    tens = {}
    for name in _W_FIELDS:
        a = w[name]
        t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
        if name.startswith("w_"):
            tb = t.to(torch.bfloat16)
            if not torch.equal(tb.to(torch.float32), t):
                raise ValueError(f"{name}: values are not bf16-representable")
            t = tb
        tens[name] = t.to(device).contiguous()
    cs = BlockWeights(**{n: tens[n].data_ptr() for n in _W_FIELDS})
    return DeviceBlock(tens, cs)


def chorus_dit_block_workspace_bytes(shape: BlockShape, Ls: int) -> int:
    return load().chorus_dit_block_workspace_bytes(C.byref(shape), int(Ls))


def chorus_dit_block_step(shape: BlockShape, weights: DeviceBlock, x, Ls, token_idx, text_ctx, t_mod,
                          tgaa_key_scale=None, gamma_o=1.0, ws=None):
    lib = load()
    _chk(x, torch.float32, "x")
    _chk(token_idx, torch.int32, "token_idx")
    _chk(text_ctx, torch.bfloat16, "text_ctx", (shape.Lt, shape.D))
    _chk(t_mod, torch.float32, "t_mod", (6, shape.D))
    _chk(tgaa_key_scale, torch.float32, "tgaa_key_scale", (shape.Lt,))
    if x.shape[-1] != shape.D or x.shape[0] < Ls:
        raise TypeError("x: wrong shape")
    if ws is None:
        ws = _ws(lib.chorus_dit_block_workspace_bytes(C.byref(shape), int(Ls)), x.device)
    _status("chorus_dit_block_step",
            lib.chorus_dit_block_step(C.byref(shape), C.byref(weights.cstruct), _p(x), int(Ls), _p(token_idx),
                                      _p(text_ctx), _p(t_mod), _p(tgaa_key_scale), float(gamma_o), _p(ws), ws.numel(),
                                      _stream()))
    return x


def chorus_text_kv_project(shape: BlockShape, weights: DeviceBlock, text_ctx, text_kv=None):
    """Projects one block's text keys / values; returns the uint8 device buffer that chorus_dit_block_step_kv takes."""
    lib = load()
    _chk(text_ctx, torch.bfloat16, "text_ctx", (shape.Lt, shape.D))
    need = lib.chorus_text_kv_bytes(C.byref(shape))
    if text_kv is None:
        text_kv = torch.empty(need, dtype=torch.uint8, device=text_ctx.device)
    _chk(text_kv, torch.uint8, "text_kv", (need,))
    ws = _ws(lib.chorus_text_kv_workspace_bytes(C.byref(shape)), text_ctx.device)
    _status("chorus_text_kv_project", lib.chorus_text_kv_project(C.byref(shape), C.byref(weights.cstruct), _p(text_ctx),
                                                                 _p(text_kv), _p(ws), ws.numel(), _stream()))
    return text_kv


def chorus_dit_block_step_kv(shape: BlockShape, weights: DeviceBlock, x, Ls, token_idx, text_kv, t_mod,
                             tgaa_key_scale=None, gamma_o=1.0, ws=None):
    lib = load()
    _chk(x, torch.float32, "x")
    _chk(token_idx, torch.int32, "token_idx")
    _chk(text_kv, torch.uint8, "text_kv", (lib.chorus_text_kv_bytes(C.byref(shape)),))
    _chk(t_mod, torch.float32, "t_mod", (6, shape.D))
    _chk(tgaa_key_scale, torch.float32, "tgaa_key_scale", (shape.Lt,))
    if x.shape[-1] != shape.D or x.shape[0] < Ls:
        raise TypeError("x: wrong shape")
    if ws is None:
        ws = _ws(lib.chorus_dit_block_workspace_bytes(C.byref(shape), int(Ls)), x.device)
    _status("chorus_dit_block_step_kv",
            lib.chorus_dit_block_step_kv(C.byref(shape), C.byref(weights.cstruct), _p(x), int(Ls), _p(token_idx),
                                         _p(text_kv), _p(t_mod), _p(tgaa_key_scale), float(gamma_o), _p(ws), ws.numel(),
                                         _stream()))
    return x


# ------------------------------------------------------- single operations

EPI_BF16, EPI_GELU_BF16, EPI_F32, EPI_RESID = 0, 1, 2, 3
PROF_SELF_ATTN, PROF_CROSS_ATTN, PROF_GEMM, PROF_NORM = 0, 1, 2, 3


def chorus_gemm_bf16(A, W, epilogue, out, bias=None, gate0=None, gate1=None, scale=1.0, M=None, kernel=0):
    lib = load()
    _chk(A, torch.bfloat16, "A")
    _chk(W, torch.bfloat16, "W")
    M = A.shape[0] if M is None else M
    N, K = W.shape
    if A.shape[1] != K:
        raise TypeError("A/W inner dimensions differ")
    want = torch.float32 if epilogue in (EPI_F32, EPI_RESID) else torch.bfloat16
    _chk(out, want, "out")
    if out.shape[-1] != N or out.shape[0] < M:
        raise TypeError("out: wrong shape")
    for n, t in (("bias", bias), ("gate0", gate0), ("gate1", gate1)):
        _chk(t, torch.float32, n, (N,))
    if kernel:
        _status("chorus_gemm_bf16_kernel", lib.chorus_gemm_bf16_kernel(_p(A), _p(W), M, N, K, epilogue, _p(out), _p(bias),
                                                                       _p(gate0), _p(gate1), float(scale), int(kernel),
                                                                       _stream()))
        return out
    _status("chorus_gemm_bf16", lib.chorus_gemm_bf16(_p(A), _p(W), M, N, K, epilogue, _p(out), _p(bias), _p(gate0),
                                                     _p(gate1), float(scale), _stream()))
    return out


def chorus_ln_modulate(x, out, mul0, mul1, add0, add1, plus_one):
    lib = load()
    _chk(x, torch.float32, "x")
    _chk(out, torch.bfloat16, "out", x.shape)
    L, D = x.shape
    for n, t in (("mul0", mul0), ("mul1", mul1), ("add0", add0), ("add1", add1)):
        _chk(t, torch.float32, n, (D,))
    _status("chorus_ln_modulate", lib.chorus_ln_modulate(_p(x), _p(out), L, D, _p(mul0), _p(mul1), _p(add0), _p(add1),
                                                         int(plus_one), _stream()))
    return out


def chorus_qk_norm_rope(inp, col0, gain, out, L, H, dh, token_idx, grid, rope, out_scale=1.0):
    """inp: bf16 [L, ld]; the D = H*dh columns starting at col0 are normalised (and multiplied by out_scale)."""
    lib = load()
    _chk(inp, torch.bfloat16, "inp")
    _chk(out, torch.bfloat16, "out")
    _chk(gain, torch.float32, "gain", (H * dh,))
    _chk(token_idx, torch.int32, "token_idx")
    ld = inp.shape[1]
    Lpad = out.shape[1]
    if tuple(out.shape) != (H, Lpad, dh) or col0 + H * dh > ld or inp.shape[0] < L:
        raise TypeError("shape mismatch")
    ptr = C.c_void_p(inp.data_ptr() + 2 * col0)
    _status("chorus_qk_norm_rope", lib.chorus_qk_norm_rope(ptr, ld, _p(gain), _p(out), L, Lpad, H, dh, _p(token_idx),
                                                           grid[0], grid[1], grid[2], int(rope), float(out_scale), _stream()))
    return out


def chorus_v_transpose(inp, col0, out, L):
    lib = load()
    _chk(inp, torch.bfloat16, "inp")
    _chk(out, torch.bfloat16, "out")
    D, Lpad = out.shape
    ld = inp.shape[1]
    if col0 + D > ld or inp.shape[0] < L:
        raise TypeError("shape mismatch")
    ptr = C.c_void_p(inp.data_ptr() + 2 * col0)
    _status("chorus_v_transpose", lib.chorus_v_transpose(ptr, ld, _p(out), L, Lpad, D, _stream()))
    return out


def chorus_attention(Q, K, Vt, O, col_scale, Lq, Lk, variant=0):
    lib = load()
    for n, t in (("Q", Q), ("K", K), ("Vt", Vt), ("O", O)):
        _chk(t, torch.bfloat16, n)
    H, LqPad, dh = Q.shape
    LkPad = K.shape[1]
    if K.shape[0] != H or K.shape[2] != dh or tuple(Vt.shape) != (H * dh, LkPad) or O.shape[1] != H * dh or O.shape[0] < Lq:
        raise TypeError("shape mismatch")
    _chk(col_scale, torch.float32, "col_scale")
    if col_scale is not None and col_scale.numel() < Lk:
        raise TypeError("col_scale too short")
    _status("chorus_attention", lib.chorus_attention(_p(Q), _p(K), _p(Vt), _p(O), _p(col_scale), Lq, Lk, LqPad, LkPad,
                                                     H, dh, int(variant), _stream()))
    return O


# ------------------------------------------------------------- step glue

@dataclass
class DeviceGlue:
    tensors: dict
    cstruct: GlueWeights


def upload_glue_weights(gw: dict, device="cuda") -> DeviceGlue:
    import numpy as np
    tens = {}
    for name, a in gw.items():
        t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
        if name.startswith("w_"):
            tb = t.to(torch.bfloat16)
            if not torch.equal(tb.to(torch.float32), t):
                raise ValueError(f"{name}: values are not bf16-representable")
            t = tb
        tens[name] = t.to(device).contiguous()
    cs = GlueWeights(**{n: tens[n].data_ptr() for n in ("w_patch", "b_patch", "w_head", "b_head", "head_table")})
    return DeviceGlue(tens, cs)


def make_model_shape(bshape: BlockShape, latent_shape, patch_hw=(2, 2), n_blocks=1):
    Cc, T, Hl, Wl = latent_shape
    return ModelShape(bshape, Cc, T, Hl, Wl, patch_hw[0], patch_hw[1], n_blocks)


def chorus_text_project(text, glue: DeviceGlue, ctx=None, ws=None):
    lib = load()
    _chk(text, torch.bfloat16, "text")
    Lt, td = text.shape
    D = glue.tensors["w_text1"].shape[0]
    if ctx is None:
        ctx = torch.empty(Lt, D, dtype=torch.bfloat16, device=text.device)
    if ws is None:
        ws = _ws(lib.chorus_text_project_workspace_bytes(Lt, D), text.device)
    t = glue.tensors
    _status("chorus_text_project", lib.chorus_text_project(_p(text), Lt, td, D, _p(t["w_text1"]), _p(t["b_text1"]),
                                                           _p(t["w_text2"]), _p(t["b_text2"]), _p(ctx), _p(ws),
                                                           ws.numel(), _stream()))
    return ctx


def chorus_patch_embed(latent, token_idx, Ls, glue: DeviceGlue, D, x, patch_hw=(2, 2), ws=None):
    lib = load()
    _chk(latent, torch.float32, "latent")
    _chk(token_idx, torch.int32, "token_idx")
    _chk(x, torch.float32, "x")
    Cc, T, Hl, Wl = latent.shape
    P = Cc * patch_hw[0] * patch_hw[1]
    if ws is None:
        ws = _ws(lib.chorus_glue_workspace_bytes(D, P, Ls), latent.device)
    _status("chorus_patch_embed", lib.chorus_patch_embed(_p(latent), Cc, T, Hl, Wl, patch_hw[0], patch_hw[1],
                                                         _p(token_idx), Ls, C.byref(glue.cstruct), D, _p(x), _p(ws),
                                                         ws.numel(), _stream()))
    return x


def chorus_head_update(latent, x, Ls, token_idx, glue: DeviceGlue, t_head, dsigma, patch_hw=(2, 2), ws=None):
    lib = load()
    _chk(latent, torch.float32, "latent")
    _chk(x, torch.float32, "x")
    _chk(token_idx, torch.int32, "token_idx")
    D = x.shape[1]
    _chk(t_head, torch.float32, "t_head", (2, D))
    Cc, T, Hl, Wl = latent.shape
    P = Cc * patch_hw[0] * patch_hw[1]
    if ws is None:
        ws = _ws(lib.chorus_glue_workspace_bytes(D, P, Ls), latent.device)
    _status("chorus_head_update", lib.chorus_head_update(_p(latent), _p(x), Ls, _p(token_idx), C.byref(glue.cstruct),
                                                         _p(t_head), float(dsigma), D, Cc, T, Hl, Wl, patch_hw[0],
                                                         patch_hw[1], _p(ws), ws.numel(), _stream()))
    return latent


def chorus_head_update_region(latent, x, Ls, token_idx, glue: DeviceGlue, t_head, dsigma, SL=None, mask_edit=None,
                              patch_hw=(2, 2), ws=None):
    """chorus_head_update with Eq. 6 on the selected tokens in the same pass (SL, mask_edit both given or both None)."""
    lib = load()
    _chk(latent, torch.float32, "latent")
    _chk(x, torch.float32, "x")
    _chk(token_idx, torch.int32, "token_idx")
    D = x.shape[1]
    _chk(t_head, torch.float32, "t_head", (2, D))
    _chk(SL, torch.float32, "SL", tuple(latent.shape))
    _chk(mask_edit, torch.uint8, "mask_edit")
    Cc, T, Hl, Wl = latent.shape
    P = Cc * patch_hw[0] * patch_hw[1]
    if ws is None:
        ws = _ws(lib.chorus_glue_workspace_bytes(D, P, Ls), latent.device)
    _status("chorus_head_update_region",
            lib.chorus_head_update_region(_p(latent), _p(x), Ls, _p(token_idx), C.byref(glue.cstruct), _p(t_head),
                                          float(dsigma), _p(SL), _p(mask_edit), D, Cc, T, Hl, Wl, patch_hw[0], patch_hw[1],
                                          _p(ws), ws.numel(), _stream()))
    return latent


def chorus_sampler_coefficients(sigmas, i, order=2) -> SamplerCoef:
    """Weights of step i (sigmas[i] -> sigmas[i + 1]) of the DPM-Solver++ update; host arithmetic in the library."""
    n_steps = len(sigmas) - 1
    sig = (C.c_float * (n_steps + 1))(*[float(v) for v in sigmas])
    out = SamplerCoef()
    _status("chorus_sampler_coefficients", load().chorus_sampler_coefficients(sig, n_steps, int(i), int(order),
                                                                              C.byref(out)))
    return out


def chorus_head_update_solver(latent, x, Ls, token_idx, glue: DeviceGlue, t_head, coef: SamplerCoef, x0_prev=None,
                              hist=None, x_uncond=None, guidance=1.0, SL=None, mask_edit=None, patch_hw=(2, 2), ws=None):
    lib = load()
    _chk(latent, torch.float32, "latent")
    _chk(x, torch.float32, "x")
    _chk(x_uncond, torch.float32, "x_uncond", x.shape)
    _chk(token_idx, torch.int32, "token_idx")
    D = x.shape[1]
    _chk(t_head, torch.float32, "t_head", (2, D))
    _chk(x0_prev, torch.float32, "x0_prev", latent.shape)
    _chk(SL, torch.float32, "SL", latent.shape)
    _chk(hist, torch.uint8, "hist")
    _chk(mask_edit, torch.uint8, "mask_edit")
    Cc, T, Hl, Wl = latent.shape
    P = Cc * patch_hw[0] * patch_hw[1]
    if ws is None:
        ws = _ws(lib.chorus_head_solver_workspace_bytes(D, P, Ls, int(x_uncond is not None)), latent.device)
    _status("chorus_head_update_solver",
            lib.chorus_head_update_solver(_p(latent), _p(x), _p(x_uncond), float(guidance), Ls, _p(token_idx),
                                          C.byref(glue.cstruct), _p(t_head), C.byref(coef), _p(x0_prev), _p(hist), _p(SL),
                                          _p(mask_edit), D, Cc, T, Hl, Wl, patch_hw[0], patch_hw[1], _p(ws), ws.numel(),
                                          _stream()))
    return latent


def block_array(blocks):
    """Host array of chorus_block_weights structs from a list of DeviceBlock."""
    arr = (BlockWeights * max(len(blocks), 1))()
    for i, b in enumerate(blocks):
        arr[i] = b.cstruct
    return arr


def chorus_denoise_step_workspace_bytes(model: ModelShape, Ls: int) -> int:
    return load().chorus_denoise_step_workspace_bytes(C.byref(model), int(Ls))


def chorus_denoise_step(model: ModelShape, blocks_arr, glue: DeviceGlue, latent, token_idx, Ls, text_ctx, t_mod, t_head,
                        tgaa_key_scale=None, gamma_o=1.0, dsigma=0.0, SL=None, mask_edit=None, ws=None):
    lib = load()
    D = model.block.D
    _chk(latent, torch.float32, "latent", (model.C, model.T, model.Hl, model.Wl))
    _chk(SL, torch.float32, "SL", latent.shape)
    _chk(token_idx, torch.int32, "token_idx")
    _chk(text_ctx, torch.bfloat16, "text_ctx", (model.block.Lt, D))
    _chk(t_mod, torch.float32, "t_mod", (6, D))
    _chk(t_head, torch.float32, "t_head", (2, D))
    _chk(tgaa_key_scale, torch.float32, "tgaa_key_scale", (model.block.Lt,))
    _chk(mask_edit, torch.uint8, "mask_edit")
    if ws is None:
        ws = _ws(lib.chorus_denoise_step_workspace_bytes(C.byref(model), int(Ls)), latent.device)
    _status("chorus_denoise_step",
            lib.chorus_denoise_step(C.byref(model), blocks_arr, C.byref(glue.cstruct), _p(latent), _p(token_idx), int(Ls),
                                    _p(text_ctx), _p(t_mod), _p(t_head), _p(tgaa_key_scale), float(gamma_o),
                                    float(dsigma), _p(SL), _p(mask_edit), _p(ws), ws.numel(), _stream()))
    return latent


def chorus_model_text_kv_project(model: ModelShape, blocks_arr, text_ctx, text_kv=None):
    """Text keys / values of every block for one request (uint8 device buffer for chorus_denoise_step_kv)."""
    lib = load()
    _chk(text_ctx, torch.bfloat16, "text_ctx", (model.block.Lt, model.block.D))
    need = lib.chorus_model_text_kv_bytes(C.byref(model))
    if text_kv is None:
        text_kv = torch.empty(max(need, 1), dtype=torch.uint8, device=text_ctx.device)
    ws = _ws(lib.chorus_text_kv_workspace_bytes(C.byref(model.block)), text_ctx.device)
    _status("chorus_model_text_kv_project", lib.chorus_model_text_kv_project(C.byref(model), blocks_arr, _p(text_ctx),
                                                                             _p(text_kv), _p(ws), ws.numel(), _stream()))
    return text_kv


def chorus_denoise_step_kv(model: ModelShape, blocks_arr, glue: DeviceGlue, latent, token_idx, Ls, text_kv, t_mod, t_head,
                           tgaa_key_scale=None, gamma_o=1.0, dsigma=0.0, SL=None, mask_edit=None, ws=None):
    lib = load()
    D = model.block.D
    _chk(latent, torch.float32, "latent", (model.C, model.T, model.Hl, model.Wl))
    _chk(SL, torch.float32, "SL", latent.shape)
    _chk(token_idx, torch.int32, "token_idx")
    _chk(text_kv, torch.uint8, "text_kv")
    _chk(t_mod, torch.float32, "t_mod", (6, D))
    _chk(t_head, torch.float32, "t_head", (2, D))
    _chk(tgaa_key_scale, torch.float32, "tgaa_key_scale", (model.block.Lt,))
    _chk(mask_edit, torch.uint8, "mask_edit")
    if text_kv.numel() < lib.chorus_model_text_kv_bytes(C.byref(model)):
        raise TypeError("text_kv: too small")
    if ws is None:
        ws = _ws(lib.chorus_denoise_step_workspace_bytes(C.byref(model), int(Ls)), latent.device)
    _status("chorus_denoise_step_kv",
            lib.chorus_denoise_step_kv(C.byref(model), blocks_arr, C.byref(glue.cstruct), _p(latent), _p(token_idx), int(Ls),
                                       _p(text_kv), _p(t_mod), _p(t_head), _p(tgaa_key_scale), float(gamma_o),
                                       float(dsigma), _p(SL), _p(mask_edit), _p(ws), ws.numel(), _stream()))
    return latent


def chorus_denoise_step_solver(model: ModelShape, blocks_arr, glue: DeviceGlue, latent, token_idx, Ls, text_kv, t_mod,
                               t_head, coef: SamplerCoef, x0_prev=None, hist=None, text_kv_uncond=None, guidance=1.0,
                               tgaa_key_scale=None, gamma_o=1.0, SL=None, mask_edit=None, outside_is_source=False,
                               ws=None):
    lib = load()
    D = model.block.D
    _chk(latent, torch.float32, "latent", (model.C, model.T, model.Hl, model.Wl))
    _chk(SL, torch.float32, "SL", latent.shape)
    _chk(x0_prev, torch.float32, "x0_prev", latent.shape)
    _chk(token_idx, torch.int32, "token_idx")
    _chk(text_kv, torch.uint8, "text_kv")
    _chk(text_kv_uncond, torch.uint8, "text_kv_uncond")
    _chk(t_mod, torch.float32, "t_mod", (6, D))
    _chk(t_head, torch.float32, "t_head", (2, D))
    _chk(tgaa_key_scale, torch.float32, "tgaa_key_scale", (model.block.Lt,))
    Ltok = model.T * (model.Hl // model.ph) * (model.Wl // model.pw)
    _chk(mask_edit, torch.uint8, "mask_edit", (Ltok,))
    _chk(hist, torch.uint8, "hist", (Ltok,))
    need = lib.chorus_model_text_kv_bytes(C.byref(model))
    for kv in (text_kv, text_kv_uncond):
        if kv is not None and kv.numel() < need:
            raise TypeError("text_kv: too small")
    cfg = int(text_kv_uncond is not None)
    if ws is None:
        ws = _ws(lib.chorus_denoise_step_solver_workspace_bytes(C.byref(model), int(Ls), cfg), latent.device)
    _status("chorus_denoise_step_solver",
            lib.chorus_denoise_step_solver(C.byref(model), blocks_arr, C.byref(glue.cstruct), _p(latent), _p(token_idx),
                                           int(Ls), _p(text_kv), _p(text_kv_uncond), float(guidance), _p(t_mod),
                                           _p(t_head), _p(tgaa_key_scale), float(gamma_o), C.byref(coef), _p(x0_prev),
                                           _p(hist), _p(SL), _p(mask_edit), int(bool(outside_is_source)), _p(ws),
                                           ws.numel(), _stream()))
    return latent


def chorus_stage1_copy(latent, SL):
    _chk(latent, torch.float32, "latent")
    _chk(SL, torch.float32, "SL", latent.shape)
    _status("chorus_stage1_copy", load().chorus_stage1_copy(_p(latent), _p(SL), latent.numel(), _stream()))
    return latent


# ---------------------------------------------------------------- region masks

def chorus_mask_pooled_extent(n: int, k: int, lead: int = 0) -> int:
    r = load().chorus_mask_pooled_extent(int(n), int(k), int(lead))
    if r < 0:
        _status("chorus_mask_pooled_extent", r)
    return r


def chorus_mask_project(key_masks, frame_key, Tp, window, t_lead=0, out=None):
    """key_masks uint8 [Kf, Hp, Wp], frame_key int32 [Tp] or None -> uint8 [To, Ho, Wo]."""
    lib = load()
    _chk(key_masks, torch.uint8, "key_masks")
    _chk(frame_key, torch.int32, "frame_key", (Tp,))
    Kf, Hp, Wp = key_masks.shape
    kt, kh, kw = (int(v) for v in window)
    shape = (chorus_mask_pooled_extent(Tp, kt, t_lead), chorus_mask_pooled_extent(Hp, kh), chorus_mask_pooled_extent(Wp, kw))
    if out is None:
        out = torch.empty(shape, dtype=torch.uint8, device=key_masks.device)
    _chk(out, torch.uint8, "out", shape)
    _status("chorus_mask_project", lib.chorus_mask_project(_p(key_masks), Kf, _p(frame_key), int(Tp), Hp, Wp, kt, kh, kw,
                                                           int(t_lead), _p(out), _stream()))
    return out


def chorus_mask_hierarchy(mask_base, r_edit, r_see, want_edit=True, want_see=True):
    """Eq. 5 on a uint8 [T, H, W] mask; returns (mask_edit, mask_see) (None where not wanted)."""
    lib = load()
    _chk(mask_base, torch.uint8, "mask_base")
    T, H, W = mask_base.shape
    edit = torch.empty_like(mask_base) if want_edit else None
    see = torch.empty_like(mask_base) if want_see else None
    re = (C.c_int32 * 3)(*[int(v) for v in r_edit]) if r_edit is not None else None
    rs = (C.c_int32 * 3)(*[int(v) for v in r_see])
    _status("chorus_mask_hierarchy", lib.chorus_mask_hierarchy(_p(mask_base), T, H, W, re, rs, _p(edit), _p(see), _stream()))
    return edit, see


def chorus_denoise_run_workspace_bytes(model: ModelShape, N: int) -> int:
    return load().chorus_denoise_run_workspace_bytes(C.byref(model), int(N))


def chorus_denoise_run(model: ModelShape, blocks_arr, glue: DeviceGlue, latent, cache_emb, cache_latents, query, tau,
                       sigmas, t_mods, t_heads, text_ctx, tdiff=None, mask_see=None, mask_edit=None, sched=None,
                       ws=None, store_slot=-1, store_after=0, solver_order=1, text_ctx_uncond=None, guidance=1.0,
                       latent_steps=None):
    """Runs one request; returns a dict with the lookup result, K1, K2 and the stage-2 token count.
    store_slot >= 0: on a miss, the query and the latent after store_after steps go into that cache entry.
    solver_order 2: DPM-Solver++ multistep update; text_ctx_uncond: classifier-free guidance with scale guidance.
    latent_steps: the depths every cache entry holds a latent for; cache_latents is then [N, len(latent_steps), ...]."""
    lib = load()
    D = model.block.D
    n_steps = len(sigmas) - 1
    N, d = cache_emb.shape
    _chk(latent, torch.float32, "latent", (model.C, model.T, model.Hl, model.Wl))
    _chk(cache_emb, torch.float32, "cache_emb")
    S = None if latent_steps is None else len(latent_steps)
    _chk(cache_latents, torch.float32, "cache_latents", ((N,) if S is None else (N, S)) + tuple(latent.shape))
    ls = None if S is None else (C.c_int32 * max(S, 1))(*[int(v) for v in latent_steps])
    _chk(query, torch.float32, "query", (d,))
    _chk(t_mods, torch.float32, "t_mods", (n_steps, 6, D))
    _chk(t_heads, torch.float32, "t_heads", (n_steps, 2, D))
    _chk(text_ctx, torch.bfloat16, "text_ctx", (model.block.Lt, D))
    _chk(text_ctx_uncond, torch.bfloat16, "text_ctx_uncond", (model.block.Lt, D))
    _chk(tdiff, torch.uint8, "tdiff", (model.block.Lt,))
    Ltok = model.T * (model.Hl // model.ph) * (model.Wl // model.pw)
    _chk(mask_see, torch.uint8, "mask_see", (Ltok,))
    _chk(mask_edit, torch.uint8, "mask_edit", (Ltok,))
    sp = None
    if sched is not None:
        dflt = dict(a1=0.25, b1=0.25, a2=0.25, b2=0.25, r3=1, Gamma_k=1.5, Gamma_o=1.5, lam=0.5, gamma_override=0.0)
        dflt.update(sched)
        sp = SchedParams(**dflt)
    sig = (C.c_float * (n_steps + 1))(*[float(v) for v in sigmas])
    rq = Request(cache_emb.data_ptr() if N else 0, cache_latents.data_ptr() if N else 0, N, d, query.data_ptr(),
                 float(tau), C.pointer(sp) if sp is not None else None, n_steps, sig, t_mods.data_ptr(),
                 t_heads.data_ptr(), text_ctx.data_ptr(), 0 if tdiff is None else tdiff.data_ptr(),
                 0 if mask_see is None else mask_see.data_ptr(), 0 if mask_edit is None else mask_edit.data_ptr(),
                 int(store_slot), int(store_after), ls, 0 if S is None else S, int(solver_order),
                 0 if text_ctx_uncond is None else text_ctx_uncond.data_ptr(), float(guidance))
    if ws is None:
        ws = _ws(lib.chorus_denoise_run_workspace_bytes(C.byref(model), N), latent.device)
    res = RunResult()
    _status("chorus_denoise_run", lib.chorus_denoise_run(C.byref(model), blocks_arr, C.byref(glue.cstruct), C.byref(rq),
                                                         _p(latent), C.byref(res), _p(ws), ws.numel(), _stream()))
    return dict(index=res.index, score=res.score, hit=bool(res.hit), K1=res.K1, K2=res.K2, Ls=res.Ls)


def prof_enable(classes=()):
    """classes: iterable of PROF_* ids to time (empty = off)."""
    mask = 0
    for c in classes:
        mask |= 1 << c
    load().chorus_prof_enable(mask)


def prof_reset():
    load().chorus_prof_reset()


def prof_read(kernel_class):
    ms, n = C.c_double(0), C.c_int32(0)
    _status("chorus_prof_read", load().chorus_prof_read(kernel_class, C.byref(ms), C.byref(n)))
    return ms.value, n.value


def chorus_mfma_ceiling(normal_data=True, mix=0, launches=20, device="cuda"):
    """Sustained TFLOP/s of a bare bf16 MFMA loop on this device (mix bit 0: operands read from LDS,
    bit 1: exp2 at the softmax ratio); see include/chorus_ops.h."""
    lib = load()
    ws = _ws(lib.chorus_mfma_ceiling_workspace_bytes(), device)
    out = C.c_double(0)
    _status("chorus_mfma_ceiling", lib.chorus_mfma_ceiling(int(bool(normal_data)), int(mix), int(launches), C.byref(out),
                                                           _p(ws), ws.numel(), _stream()))
    return out.value


class DeviceTime:
    """Device copies of the timestep-embedding weights and the struct of pointers to them."""

    def __init__(self, tw: dict, device="cuda"):
        import numpy as np
        self.tensors = {}
        for k, v in tw.items():
            a = np.ascontiguousarray(v, dtype=np.float32)
            t = torch.from_numpy(a).to(device)
            self.tensors[k] = t.to(torch.bfloat16).contiguous() if k.startswith("w_") else t
        self.freq_dim = tw["w_t1"].shape[1]
        self.D = tw["w_t1"].shape[0]
        self.cstruct = TimeWeights(*[self.tensors[n].data_ptr() for n in ("w_t1", "b_t1", "w_t2", "b_t2", "w_tp", "b_tp")])


def chorus_time_mod(t, tw: DeviceTime, t_mod=None, t_head=None, ws=None):
    """(t_mod [6, D], t_head [2, D]) of one timestep value."""
    lib = load()
    dev = tw.tensors["w_t1"].device
    D = tw.D
    if t_mod is None:
        t_mod = torch.empty(6, D, dtype=torch.float32, device=dev)
    if t_head is None:
        t_head = torch.empty(2, D, dtype=torch.float32, device=dev)
    _chk(t_mod, torch.float32, "t_mod", (6, D))
    _chk(t_head, torch.float32, "t_head", (2, D))
    if ws is None:
        ws = _ws(lib.chorus_time_mod_workspace_bytes(D, tw.freq_dim), dev)
    _status("chorus_time_mod", lib.chorus_time_mod(float(t), tw.freq_dim, D, C.byref(tw.cstruct), _p(t_mod), _p(t_head),
                                                   _p(ws), ws.numel(), _stream()))
    return t_mod, t_head
