"""Pins for the whole operator as the fp64 oracle computes it: symmetry properties, special cases that
reduce to a library routine, and the agreement of its independent routes."""
import numpy as np
import pytest

import oracle as O
from paper_2601_16622_amd import workloads as W

RNG = np.random.default_rng(4321)


def Rz(a):
    c, s = np.cos(a), np.sin(a)
    return np.array([[c, -s, 0], [s, c, 0], [0, 0, 1.0]])


def Ry(a):
    c, s = np.cos(a), np.sin(a)
    return np.array([[c, 0, s], [0, 1.0, 0], [-s, 0, c]])


def small_case(seed, L=2, C=8, H=2, B=4, lf=1, n_seg=2, per_seg=14, cutoff=3.0):
    """Random clusters, with no pair closer than 1e-3 to the cutoff sphere (the softmax normaliser changes
    discontinuously when a pair enters the neighbourhood, so symmetry checks need a margin)."""
    rng = np.random.default_rng(seed)
    while True:
        pos = np.concatenate([W.dart_throw_box(rng, per_seg, 5.0, origin=rng.uniform(-4, 4, 3)) for _ in range(n_seg)])
        pos = pos.astype(np.float64)
        seg = np.arange(n_seg + 1, dtype=np.int32) * per_seg
        d = np.linalg.norm(pos[:, None] - pos[None], axis=-1)
        if np.abs(d - cutoff).min() > 1e-3:
            break
    cfg = dict(L=L, C=C, H=H, B=B, lf=lf, cutoff=cutoff)
    N, n = pos.shape[0], (L + 1) ** 2
    h = rng.normal(size=(N, n, C))
    lim = np.sqrt(6.0 / (2 * C))
    w = {k: rng.uniform(-lim, lim, size=(L + 1, C, C)) for k in ("WQ1", "WQ2", "WK1", "WK2", "WV")}
    w["Wb"] = rng.normal(size=(H, B)) / np.sqrt(B)
    w["w_path"] = rng.uniform(0.5, 1.5, size=(L + 1, L + 1))
    return cfg, pos, seg, h, w


def rotate_features(h, L, a, b, g):
    out = np.empty_like(h)
    for l in range(L + 1):
        D = O.wigner_D_real(l, a, b, g)
        out[:, l * l:(l + 1) ** 2] = np.einsum("ab,nbc->nac", D, h[:, l * l:(l + 1) ** 2])
    return out


@pytest.mark.parametrize("mode", ["dense", "eaas"])
@pytest.mark.parametrize("lf", [1, 2])
def test_rotation_equivariance(mode, lf):
    cfg, pos, seg, h, w = small_case(1, lf=lf)
    a, b, g = RNG.uniform(-3, 3, size=3)
    R = Rz(a) @ Ry(b) @ Rz(g)
    out = O.attn_forward(cfg, pos, h, seg, w, message_mode=mode)
    out_rot = O.attn_forward(cfg, pos @ R.T, rotate_features(h, cfg["L"], a, b, g), seg, w, message_mode=mode)
    assert np.abs(out).max() > 0.1
    np.testing.assert_allclose(out_rot, rotate_features(out, cfg["L"], a, b, g), atol=1e-10)


def test_translation_invariance():
    cfg, pos, seg, h, w = small_case(2)
    out = O.attn_forward(cfg, pos, h, seg, w)
    shifted = O.attn_forward(cfg, pos + np.array([3.25, -7.5, 11.125]), h, seg, w)
    np.testing.assert_allclose(shifted, out, atol=1e-10)


def test_permutation_equivariance():
    cfg, pos, seg, h, w = small_case(3, n_seg=1, per_seg=24)
    perm = RNG.permutation(pos.shape[0])
    out = O.attn_forward(cfg, pos, h, seg, w)
    outp = O.attn_forward(cfg, pos[perm], h[perm], seg, w)
    np.testing.assert_allclose(outp, out[perm], atol=1e-11)


def test_segments_do_not_interact():
    cfg, pos, seg, h, w = small_case(4, n_seg=3, per_seg=10)
    pos[10:20] = pos[0:10] + 0.37          # overlay the second system on the first
    out = O.attn_forward(cfg, pos, h, seg, w)
    alone = O.attn_forward(cfg, pos[10:20], h[10:20], np.array([0, 10], dtype=np.int32), w)
    np.testing.assert_allclose(out[10:20], alone, atol=1e-12)


@pytest.mark.parametrize("name", ["tiny", "small", "large"])
def test_cell_list_equals_all_pairs(name):
    wl = W.by_name(name, seed=5)
    rc = np.float32(wl["cfg"]["cutoff"])
    o1, i1 = O.neighbor_list(wl["pos"], wl["seg"], rc, use_cells=False)
    o2, i2 = O.neighbor_list(wl["pos"], wl["seg"], rc, use_cells=True)
    assert np.array_equal(o1, o2) and np.array_equal(i1, i2)
    # symmetric, no self pairs, inside segments
    src = np.repeat(np.arange(len(o1) - 1), np.diff(o1))
    pairs = set(zip(src.tolist(), i1.tolist()))
    assert all((j, i) in pairs for i, j in pairs) and all(i != j for i, j in pairs)
    seg_of = np.searchsorted(wl["seg"], np.arange(wl["pos"].shape[0]), side="right")
    assert np.array_equal(seg_of[src], seg_of[i1])


def test_neighbor_predicate_is_binary32():
    """The pair test is d2 = (dx*dx + dy*dy) + dz*dz < rc*rc evaluated in binary32 on binary32 positions."""
    rng = np.random.default_rng(7)
    pos = rng.uniform(0, 6, size=(200, 3)).astype(np.float32)
    rc = np.float32(2.5)
    offs, idx = O.neighbor_list(pos, np.array([0, 200], dtype=np.int32), rc)
    dx = pos[None, :, :] - pos[:, None, :]
    sq = dx * dx
    d2 = (sq[..., 0] + sq[..., 1]) + sq[..., 2]
    assert d2.dtype == np.float32
    mask = (d2 < rc * rc) & (d2 > 0)
    assert np.array_equal(np.diff(offs), mask.sum(1))
    assert np.array_equal(idx, np.nonzero(mask)[1])


def test_density_of_the_scaling_workload():
    wl = W.box(3000, seed=1)
    offs, _ = O.neighbor_list(wl["pos"], wl["seg"], np.float32(6.0), use_cells=True)
    deg = np.diff(offs)
    assert 55 < deg.mean() < 90 and deg.max() < 140       # interior atoms see about 0.1 * 4/3 pi 6^3 = 90


def test_routes_agree():
    """Dense CG + two-pass softmax + all pairs  vs  EAAS + streaming recurrences + cell list."""
    cfg, pos, seg, h, w = small_case(6, L=3, C=6, H=3)
    ref = O.attn_forward(cfg, pos, h, seg, w)
    alt = O.attn_forward(cfg, pos, h, seg, w, message_mode="eaas", softmax_mode="stream", use_cells=True, chi=0.9)
    np.testing.assert_allclose(alt, ref, atol=1e-11)


def test_streaming_softmax_is_order_independent():
    cfg, pos, seg, h, w = small_case(8)
    offs, idx = O.neighbor_list(pos, seg, np.float32(cfg["cutoff"]))
    ref = O.attn_forward(cfg, pos, h, seg, w, nbr=(offs, idx))
    shuffled = idx.copy()
    for i in range(len(offs) - 1):
        RNG.shuffle(shuffled[offs[i]:offs[i + 1]])
    out = O.attn_forward(cfg, pos, h, seg, w, nbr=(offs, shuffled), softmax_mode="stream")
    np.testing.assert_allclose(out, ref, atol=1e-11)


def test_target_subset_matches_full_run():
    cfg, pos, seg, h, w = small_case(9)
    full = O.attn_forward(cfg, pos, h, seg, w)
    tg = np.array([3, 17, 20, 0], dtype=np.int32)
    np.testing.assert_allclose(O.attn_forward(cfg, pos, h, seg, w, targets=tg), full[tg], atol=1e-13)


def test_uniform_attention_special_case():
    """W_Q1 = 0 and Wb = 0 make every logit zero: out_i = (1/K_i) sum_j phi(d_ij) msg_ij (Eq. attn)."""
    cfg, pos, seg, h, w = small_case(10, L=2, C=4, H=2)
    w = dict(w)
    w["WQ1"] = np.zeros_like(w["WQ1"])
    w["Wb"] = np.zeros_like(w["Wb"])
    out = O.attn_forward(cfg, pos, h, seg, w)
    offs, idx = O.neighbor_list(pos, seg, np.float32(cfg["cutoff"]))
    L, C = cfg["L"], cfg["C"]
    v = np.empty_like(h)
    for l in range(L + 1):
        v[:, l * l:(l + 1) ** 2] = np.einsum("oc,nmc->nmo", w["WV"][l], h[:, l * l:(l + 1) ** 2])
    for i in range(pos.shape[0]):
        nb = idx[offs[i]:offs[i + 1]]
        acc = np.zeros((h.shape[1], C))
        for j in nb:
            r = pos[j] - pos[i]
            d = np.linalg.norm(r)
            acc += 0.5 * (1 + np.cos(np.pi * d / cfg["cutoff"])) * O.message(L, 1, w["w_path"], v[j], r, "dense")
        expect = acc / max(len(nb), 1)
        np.testing.assert_allclose(out[i], expect, atol=1e-12)


def test_scalar_case_is_masked_multihead_attention():
    """L = 0, l_f = 0: ordinary masked multi-head attention with q = (W_Q1 h)(W_Q2 h), written with dense
    torch ops (softmax from the library), gate applied after the softmax."""
    import torch
    rng = np.random.default_rng(11)
    N, C, H, B, rc = 40, 12, 3, 5, 2.5
    pos = W.dart_throw_box(rng, N, 6.0).astype(np.float64)
    seg = np.array([0, 25, N], dtype=np.int32)
    cfg = dict(L=0, C=C, H=H, B=B, lf=0, cutoff=rc)
    h = rng.normal(size=(N, 1, C))
    w = {k: rng.normal(size=(1, C, C)) / np.sqrt(C) for k in ("WQ1", "WQ2", "WK1", "WK2", "WV")}
    w["Wb"] = rng.normal(size=(H, B))
    w["w_path"] = np.array([[1.7]])
    out = O.attn_forward(cfg, pos, h, seg, w)

    x = torch.tensor(h[:, 0])
    T = {k: torch.tensor(v[0]) for k, v in w.items() if k.startswith("W") and k != "Wb"}
    q = (x @ T["WQ1"].T) * (x @ T["WQ2"].T)
    k = (x @ T["WK1"].T) * (x @ T["WK2"].T)
    v = x @ T["WV"].T
    Ch = C // H
    p = torch.tensor(pos)
    d = torch.cdist(p, p)
    seg_of = torch.tensor(np.searchsorted(seg, np.arange(N), side="right"))
    mask = (d < rc) & (d > 0) & (seg_of[:, None] == seg_of[None, :])
    mu = torch.arange(B, dtype=torch.float64) * rc / (B - 1)
    g = torch.exp(-0.5 * (B - 1) ** 2 / rc ** 2 * (d[..., None] - mu) ** 2)           # [N][N][B]
    bias = torch.einsum("ijb,hb->hij", g, torch.tensor(w["Wb"]))
    qh, kh, vh = (t.reshape(N, H, Ch).permute(1, 0, 2) for t in (q, k, v))
    s = qh @ kh.transpose(1, 2) / np.sqrt(Ch) + bias
    s = s.masked_fill(~mask, float("-inf"))
    a = torch.softmax(s, dim=-1)
    a = torch.nan_to_num(a, nan=0.0) * (0.5 * (1 + torch.cos(np.pi * d / rc)))
    ref = 1.7 * (a @ vh).permute(1, 0, 2).reshape(N, C)
    np.testing.assert_allclose(out[:, 0], ref.numpy(), atol=1e-12)


def test_isolated_atom_gets_zero():
    cfg, pos, seg, h, w = small_case(12, n_seg=1, per_seg=12)
    pos[5] += 100.0
    out = O.attn_forward(cfg, pos, h, seg, w)
    assert np.all(out[5] == 0.0) and np.abs(out[4]).max() > 0
