"""GPU parity: region-mask pipeline (key-frame propagation + max-pool projection, Eq. 5
dilation hierarchy) against the CPU oracle, through the C ABI. Byte work: bit-exact."""
import numpy as np
import pytest
import torch

import synth
from oracle import chorus_oracle as O
import paper_2604_04451_amd as P
from gpu_util import DEV, host

pytestmark = pytest.mark.gpu


def dev_u8(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint8)).to(DEV)


def _project(km, fk, Tp, win, t_lead):
    d_fk = None if fk is None else torch.from_numpy(np.asarray(fk, np.int32)).to(DEV)
    return host(P.chorus_mask_project(dev_u8(km), d_fk, Tp, win, t_lead))


@pytest.mark.parametrize("shape,radii", [
    ((4, 9, 11), [((0, 0, 0), (0, 0, 0)), ((0, 1, 1), (1, 2, 3)), ((1, 0, 2), (1, 3, 2)), ((2, 4, 5), (9, 20, 20))]),
    ((1, 1, 1), [((0, 0, 0), (1, 1, 1))]),
    ((3, 1, 300), [((0, 0, 2), (1, 0, 7))]),                       # one-row planes, several workgroups, ragged tail
    ((21, 30, 52), [((0, 1, 1), (1, 3, 3)), ((0, 2, 2), (0, 4, 4))]),  # the 480p token grid
    ((2, 3, 13000), [((0, 0, 1), (1, 1, 3))]),                     # rows too wide for the LDS kernel: per-site fallback
    ((3, 200, 96), [((1, 2, 2), (1, 9, 5))]),                      # several row strips per frame with halos
])
def test_mask_hierarchy(shape, radii):
    n = int(np.prod(shape))
    base = (synth.stream(1, f"gpu.dil.{shape}").random(shape) < max(0.01, 2.0 / n)).astype(np.uint8)
    base[base != 0] = synth.stream(1, "gpu.dil.val").integers(1, 256, int(base.sum()))   # any non-zero byte is set
    d_base = dev_u8(base)
    for r_edit, r_see in radii:
        print(f"[case] mask_hierarchy shape={shape} r={r_edit} r'={r_see}", flush=True)
        edit, see = P.chorus_mask_hierarchy(d_base, r_edit, r_see)
        o_edit, o_see = O.mask_hierarchy(base, r_edit, r_see)
        np.testing.assert_array_equal(host(edit), o_edit)
        np.testing.assert_array_equal(host(see), o_see)
        # single outputs: the same dilation through either slot
        e2, s2 = P.chorus_mask_hierarchy(d_base, None, r_see, want_edit=False)
        assert e2 is None and torch.equal(s2, see)
        e3, s3 = P.chorus_mask_hierarchy(d_base, r_edit, r_see, want_see=False)
        assert s3 is None and torch.equal(e3, edit)


def test_mask_hierarchy_blob_containment_and_ends():
    T, Hg, Wg = 21, 30, 52
    base = O.mask_maxpool(synth.pixel_key_masks(T, Hg * 4, Wg * 4, seed=2), (1, 4, 4))
    edit, see = P.chorus_mask_hierarchy(dev_u8(base), (0, 1, 1), (1, 3, 3))
    o_edit, o_see = O.mask_hierarchy(base, (0, 1, 1), (1, 3, 3))
    np.testing.assert_array_equal(host(edit), o_edit)
    np.testing.assert_array_equal(host(see), o_see)
    assert (host(edit) >= base).all() and (host(see) >= host(edit)).all()
    zero = torch.zeros((T, Hg, Wg), dtype=torch.uint8, device=DEV)
    e, s = P.chorus_mask_hierarchy(zero, (1, 2, 2), (2, 4, 4))
    assert int(e.sum()) == 0 and int(s.sum()) == 0
    e, s = P.chorus_mask_hierarchy(zero + 1, (1, 2, 2), (2, 4, 4))
    assert bool(e.all()) and bool(s.all())
    # empty grid: nothing to do, no launch
    e, s = P.chorus_mask_hierarchy(torch.zeros((0, 4, 4), dtype=torch.uint8, device=DEV), (0, 1, 1), (0, 1, 1))
    assert e.numel() == 0 and s.numel() == 0


@pytest.mark.parametrize("Tp,Hp,Wp,Kf,win,t_lead", [
    (9, 32, 48, 3, (4, 8, 8), 1),        # 16-byte rows, grouped key frames, leading frame
    (9, 32, 48, None, (4, 8, 8), 1),     # every frame its own key frame
    (8, 20, 50, 4, (2, 3, 5), 0),        # rows not a multiple of 16 bytes: byte path; ragged windows
    (5, 17, 33, 2, (4, 16, 16), 1),      # windows larger than what is left at every edge
    (3, 4, 1040, 3, (1, 2, 16), 0),      # more than 64 16-byte chunks per row
    (2, 5, 7, 2, (1, 1, 1), 0),          # identity pooling
    (6, 40, 64, 2, (8, 64, 64), 0),      # one window covers everything
])
def test_mask_project_small(Tp, Hp, Wp, Kf, win, t_lead):
    print(f"[case] mask_project Tp={Tp} Hp={Hp} Wp={Wp} Kf={Kf} win={win} lead={t_lead}", flush=True)
    km = synth.pixel_key_masks(Kf if Kf else Tp, Hp, Wp, seed=3, fill=0.05)
    km[km != 0] = 255                                                   # segmentation masks often come as 0 / 255
    fk = synth.frame_key_groups(Tp, Kf) if Kf else None
    frames = O.mask_propagate_keyframes(km, fk if Kf else np.arange(Tp))
    ref = O.mask_maxpool(frames, win, t_lead)
    got = _project(km, fk, Tp, win, t_lead)
    assert got.shape == ref.shape
    np.testing.assert_array_equal(got, ref)


def test_mask_project_edge_cases():
    # sparse isolated sites: every set site must survive, nothing else appears
    m = synth.sparse_site_mask((9, 33, 47), 6, seed=4)
    ref = O.mask_maxpool(m, (4, 8, 8), 1)
    np.testing.assert_array_equal(_project(m, None, 9, (4, 8, 8), 1), ref)
    assert ref.sum() <= 6 and ref.any()
    # a frame whose key index is outside [0, Kf) contributes nothing
    km = np.ones((2, 8, 16), np.uint8)
    fk = np.array([0, 5, -1, 1], np.int32)
    got = _project(km, fk, 4, (1, 8, 16), 0)
    np.testing.assert_array_equal(got.reshape(-1), [1, 0, 0, 1])
    # all-zero and all-one masks
    assert _project(np.zeros((3, 16, 32), np.uint8), None, 3, (2, 4, 4), 0).sum() == 0
    assert _project(np.ones((3, 16, 32), np.uint8), None, 3, (2, 4, 4), 0).all()
    # a base pointer that is not 16-byte aligned takes the byte path
    big = torch.zeros(1 + 2 * 16 * 32, dtype=torch.uint8, device=DEV)
    src = synth.sparse_site_mask((2, 16, 32), 9, seed=5)
    view = big[1:].view(2, 16, 32)
    view.copy_(torch.from_numpy(src))
    got = host(P.chorus_mask_project(view, None, 2, (1, 4, 4), 0))
    np.testing.assert_array_equal(got, O.mask_maxpool(src, (1, 4, 4)))


@pytest.mark.parametrize("name,Hp,Wp", [("wan1p3b_480p", 480, 832), ("wan14b_720p", 720, 1280)])
def test_mask_pipeline_full_shape(name, Hp, Wp):
    """Pixel-space key-frame masks of an 81-frame clip -> token grid -> (M_edit, M_see) -> token list,
    at the launch shapes of the benchmark workloads."""
    bs = synth.SHAPES[name]
    T, Hg, Wg = bs.grid
    Tp, Kf = 81, 21
    print(f"[case] mask pipeline {name}: {Kf} key frames {Hp}x{Wp}, {Tp} frames -> grid {bs.grid}", flush=True)
    km = synth.pixel_key_masks(Kf, Hp, Wp, seed=6, n_obj=2, fill=0.1)
    fk = synth.frame_key_groups(Tp, Kf)
    win = (4, Hp // Hg, Wp // Wg)
    base = P.chorus_mask_project(dev_u8(km), torch.from_numpy(fk).to(DEV), Tp, win, 1)
    assert tuple(base.shape) == (T, Hg, Wg)
    o_base = O.mask_maxpool(O.mask_propagate_keyframes(km, fk), win, 1)
    np.testing.assert_array_equal(host(base), o_base)
    edit, see = P.chorus_mask_hierarchy(base, (0, 1, 1), (1, 3, 3))
    o_edit, o_see = O.mask_hierarchy(o_base, (0, 1, 1), (1, 3, 3))
    np.testing.assert_array_equal(host(edit), o_edit)
    np.testing.assert_array_equal(host(see), o_see)
    idx, cnt = P.chorus_region_compact(see.reshape(-1))
    Ls = int(cnt.cpu()[0])
    np.testing.assert_array_equal(host(idx)[:Ls], O.region_compact(o_see.reshape(-1)))
    print(f"[info] base {o_base.mean():.3f} edit {o_edit.mean():.3f} see {o_see.mean():.3f} of the grid", flush=True)
    assert 0 < o_base.sum() < o_edit.sum() < o_see.sum() < o_see.size
