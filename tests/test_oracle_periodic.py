"""Pins for the oracle's periodic-boundary route (folded coordinates, one image per pair, translated pair vectors).
Periodic boundaries are this build's extension for the bulk simulations of the paper's Sec. 4.3; the operator itself
is unchanged, so every pin reduces the periodic result to the open-boundary oracle on an explicit set of images or
to a closed form."""
import numpy as np
import pytest

import oracle as O
from paper_2601_16622_amd import workloads as W


def grid_case(seed, n=80, lens=(10.0, 11.0, 9.5), cutoff=3.0, L=2, C=8, H=2, B=4, lf=1):
    """Atoms on a 1/64 grid inside the box (all coordinate sums below are exact in binary32), none closer than
    1e-3 to the cutoff sphere through any image."""
    rng = np.random.default_rng(seed)
    lens = np.asarray(lens)
    while True:
        pos = np.round(rng.uniform(0, 1, size=(n, 3)) * lens * 64) / 64
        pos = np.minimum(pos, lens - 1 / 64)
        d = pos[:, None, :] - pos[None, :, :]
        d -= lens * np.round(d / lens)
        r = np.linalg.norm(d, axis=-1)
        r[np.arange(n), np.arange(n)] = 1.0
        if r.min() > 0.5 and np.abs(r - cutoff).min() > 1e-3:
            break
    cfg = dict(L=L, C=C, H=H, B=B, lf=lf, cutoff=cutoff)
    nn = (L + 1) ** 2
    h = rng.normal(size=(n, nn, C))
    lim = np.sqrt(6.0 / (2 * C))
    w = {k: rng.uniform(-lim, lim, size=(L + 1, C, C)) for k in ("WQ1", "WQ2", "WK1", "WK2", "WV")}
    w["Wb"] = rng.normal(size=(H, B)) / np.sqrt(B)
    w["w_path"] = rng.uniform(0.5, 1.5, size=(L + 1, L + 1))
    seg = np.array([0, n], dtype=np.int32)
    return cfg, pos, seg, h, w, np.asarray([lens], dtype=np.float32)


def replicate(pos, h, lens, periodic=(True, True, True)):
    """The 27 (or fewer) translated copies of a system as one open system; copy 0 is the original."""
    rng = [(0, -1, 1) if p else (0,) for p in periodic]
    shifts = [(a, b, c) for a in rng[0] for b in rng[1] for c in rng[2]]
    P = np.concatenate([pos + np.asarray(s) * lens for s in shifts])
    Hh = np.concatenate([h] * len(shifts))
    return P, Hh, len(shifts)


@pytest.mark.parametrize("lf", [1, 2])
def test_periodic_equals_open_system_of_explicit_images(lf):
    cfg, pos, seg, h, w, box = grid_case(3, lf=lf)
    n = pos.shape[0]
    out = O.attn_forward(cfg, pos, h, seg, w, box=box)
    P, Hh, copies = replicate(pos, h, box[0].astype(np.float64))
    ref = O.attn_forward(cfg, P, Hh, np.array([0, n * copies], dtype=np.int32), w, targets=np.arange(n))
    assert np.abs(ref).max() > 0.1
    np.testing.assert_allclose(out, ref, atol=1e-11)
    # and the neighbour sets: same atoms (modulo the copy), same degree
    off, idx, shift = O.neighbor_list_periodic(pos, seg, cfg["cutoff"], box)
    roff, ridx = O.neighbor_list(P, np.array([0, n * copies], dtype=np.int32), np.float32(cfg["cutoff"]))
    crossing = 0
    for i in range(n):
        mine = sorted(idx[off[i]:off[i + 1]].tolist())
        theirs = sorted((ridx[roff[i]:roff[i + 1]] % n).tolist())
        assert mine == theirs
        crossing += int(np.any(shift[off[i]:off[i + 1]] != 0, axis=1).sum())
    assert crossing > n   # the case does exercise images (about a third of all edges cross a face)


def test_slab_with_one_open_axis_equals_explicit_images():
    cfg, pos, seg, h, w, box = grid_case(5)
    box[0, 2] = 0.0
    n = pos.shape[0]
    out = O.attn_forward(cfg, pos, h, seg, w, box=box)
    lens = np.array([box[0, 0], box[0, 1], 0.0], dtype=np.float64)
    P, Hh, copies = replicate(pos, h, lens, periodic=(True, True, False))
    assert copies == 9
    ref = O.attn_forward(cfg, P, Hh, np.array([0, n * copies], dtype=np.int32), w, targets=np.arange(n))
    np.testing.assert_allclose(out, ref, atol=1e-11)


def test_large_box_reduces_to_open_boundaries():
    cfg, pos, seg, h, w, _ = grid_case(7)
    box = np.full((1, 3), 64.0, dtype=np.float32)   # nothing reaches across: extent 11 + cutoff 3 < 64 - 11
    out = O.attn_forward(cfg, pos, h, seg, w, box=box)
    ref = O.attn_forward(cfg, pos, h, seg, w)
    np.testing.assert_allclose(out, ref, atol=1e-12)
    off, idx, shift = O.neighbor_list_periodic(pos, seg, cfg["cutoff"], box)
    roff, ridx = O.neighbor_list(pos, seg, np.float32(cfg["cutoff"]))
    assert np.array_equal(off, roff) and np.array_equal(idx, ridx) and not shift.any()


def test_invariance_under_lattice_translations_of_single_atoms_and_of_the_whole_system():
    cfg, pos, seg, h, w, box = grid_case(11)
    lens = box[0].astype(np.float64)
    out = O.attn_forward(cfg, pos, h, seg, w, box=box)
    rng = np.random.default_rng(0)
    hopped = pos + rng.integers(-3, 4, size=pos.shape) * lens          # every atom by its own lattice vector
    np.testing.assert_allclose(O.attn_forward(cfg, hopped, h, seg, w, box=box), out, atol=1e-11)
    moved = pos + np.array([37 / 64, -5.25, 123 / 64])                  # rigid shift (exact on the grid), then folded
    np.testing.assert_allclose(O.attn_forward(cfg, moved, h, seg, w, box=box), out, atol=1e-11)
    folded = O.wrap_positions(moved, seg, box)
    assert (folded >= 0).all() and (folded < box[0]).all()
    assert np.array_equal(O.wrap_positions(folded, seg, box), folded)   # idempotent
    k = (moved - folded.astype(np.float64)) / lens
    np.testing.assert_allclose(k, np.round(k), atol=1e-6)               # differs by whole box lengths only


def test_a_pair_across_the_boundary_by_hand():
    """Two atoms 1.0 apart through the x face and nothing else: each sees the other, with opposite images."""
    box = np.array([[12.0, 12.0, 12.0]], dtype=np.float32)
    pos = np.array([[0.25, 6.0, 6.0], [11.25, 6.0, 6.0], [6.0, 6.0, 1.0]])
    seg = np.array([0, 3], dtype=np.int32)
    off, idx, shift = O.neighbor_list_periodic(pos, seg, 3.0, box)
    assert off.tolist() == [0, 1, 2, 2]
    assert idx.tolist() == [1, 0]
    assert shift.tolist() == [[-1, 0, 0], [1, 0, 0]]
    t = O.edge_translations(seg, box, off, shift)
    assert t.tolist() == [[-12.0, 0, 0], [12.0, 0, 0]]
    # the operator on this pair equals the open pair at distance 1 along -x / +x
    cfg = dict(L=1, C=4, H=1, B=4, lf=1, cutoff=3.0)
    rng = np.random.default_rng(2)
    h = rng.normal(size=(3, 4, 4))
    w = {k: rng.normal(size=(2, 4, 4)) for k in ("WQ1", "WQ2", "WK1", "WK2", "WV")}
    w["Wb"] = rng.normal(size=(1, 4))
    w["w_path"] = np.ones((2, 2))
    out = O.attn_forward(cfg, pos, h, seg, w, box=box)
    open_pos = np.array([[0.25, 6.0, 6.0], [-0.75, 6.0, 6.0], [6.0, 6.0, 1.0]])
    ref = O.attn_forward(cfg, open_pos, h, seg, w)
    np.testing.assert_allclose(out, ref, atol=1e-12)
    assert np.abs(out[:2]).max() > 1e-3 and not out[2].any()


def test_neighbour_relation_is_symmetric_with_opposite_images():
    wl = W.periodic_boxes((150, 90), seed=3, L=1, C=8, H=1, cutoff=4.0)
    off, idx, shift = O.neighbor_list_periodic(wl["pos"], wl["seg"], 4.0, wl["box"])
    edges = {}
    for i in range(len(off) - 1):
        for e in range(off[i], off[i + 1]):
            edges[(i, int(idx[e]))] = tuple(int(x) for x in shift[e])
    assert len(edges) == len(idx) > 0
    for (i, j), s in edges.items():
        assert edges[(j, i)] == tuple(-x for x in s)
    assert any(any(s) for s in edges.values())


def test_full_fcc_crystal_has_54_neighbours_everywhere_and_its_odd_filter_output_vanishes():
    """Closed forms: shells of 12, 6, 24, 12 sites inside 6 A for a = 3.8.  Every site is a centre of inversion, so
    with equal features on all atoms the logits of j and of its mirror image agree and the degree-1 (odd) filter
    sums to zero; with distinct features it does not."""
    wl = W.periodic_fcc(5, L=1, C=8, H=2, B=4, dtype="f32")
    off, idx, shift = O.neighbor_list_periodic(wl["pos"], wl["seg"], 6.0, wl["box"])
    assert np.all(np.diff(off) == 54)
    cfg = {k: wl["cfg"][k] for k in ("L", "C", "H", "B", "lf", "cutoff")}
    targets = np.arange(0, 500, 37)
    h = np.broadcast_to(wl["h"][:1], wl["h"].shape).copy()
    out = O.attn_forward(cfg, wl["pos"], h, wl["seg"], wl["weights"], box=wl["box"], nbr=(off, idx, shift),
                         targets=targets)
    assert np.abs(out).max() < 1e-6      # binary32 lattice coordinates: exact up to their rounding
    out = O.attn_forward(cfg, wl["pos"], wl["h"], wl["seg"], wl["weights"], box=wl["box"], nbr=(off, idx, shift),
                         targets=targets)
    assert np.abs(out).max() > 1e-2


def test_cap_with_images_keeps_the_nearest():
    wl = W.periodic_fcc(5, L=1, C=8, H=2, B=4, dtype="f32")
    off, idx, shift = O.neighbor_list_periodic(wl["pos"], wl["seg"], 6.0, wl["box"])
    folded = O.wrap_positions(wl["pos"], wl["seg"], wl["box"])
    tr = O.edge_translations(wl["seg"], wl["box"], off, shift)
    coff, cidx, kept = O.cap_neighbors(folded, off, idx, 18, translation=tr)
    assert np.all(np.diff(coff) == 18)       # the two nearest shells, 12 + 6
    d = np.linalg.norm(folded[cidx].astype(np.float64) + tr[kept] - np.repeat(folded, 18, axis=0), axis=1)
    assert d.max() < 3.8 + 1e-4
    assert np.array_equal(idx[kept], cidx)
