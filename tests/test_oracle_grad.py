"""Pins for the gradient reference (oracle/grad.py): its forward value against the C oracle, its gradients against
central differences of the C oracle (an independent program), and the invariances a gradient must have."""
import numpy as np
import pytest

import oracle as O
from oracle import grad as G
from test_oracle_operator import small_case


def case(seed, **kw):
    cfg, pos, seg, h, w = small_case(seed, **kw)
    nbr = O.neighbor_list(pos, seg, np.float32(cfg["cutoff"]))
    go = np.random.default_rng(seed + 100).normal(size=h.shape)
    return cfg, pos, seg, h, w, nbr, go


def loss_c(cfg, pos, h, seg, w, nbr, go):
    return float((O.attn_forward(cfg, pos, h, seg, w, nbr=nbr) * go).sum())


@pytest.mark.parametrize("L,H", [(1, 1), (2, 2), (3, 2)])
def test_forward_of_the_differentiable_route_equals_the_c_oracle(L, H):
    cfg, pos, seg, h, w, nbr, go = case(5 + L, L=L, H=H)
    out, _ = G.attn_backward(cfg, pos, h, w, nbr, go, wrt=())
    ref = O.attn_forward(cfg, pos, h, seg, w, nbr=nbr)
    assert np.abs(ref).max() > 0.1
    np.testing.assert_allclose(out, ref, atol=1e-12)


def test_gradients_match_central_differences_of_the_c_oracle():
    cfg, pos, seg, h, w, nbr, go = case(3, L=2, C=4, H=2, per_seg=9)
    names = ("pos", "h", "WQ1", "WQ2", "WK1", "WK2", "WV", "Wb", "w_path")
    _, g = G.attn_backward(cfg, pos, h, w, nbr, go, wrt=names)
    rng = np.random.default_rng(0)
    eps = 1e-6
    for name in names:
        base = pos if name == "pos" else h if name == "h" else w[name]
        assert np.abs(g[name]).max() > 1e-6, name
        flat = rng.choice(base.size, size=min(12, base.size), replace=False)
        for f in flat:
            def at(delta):
                x = base.copy()
                x.reshape(-1)[f] += delta
                if name == "pos":
                    return loss_c(cfg, x, h, seg, w, nbr, go)
                if name == "h":
                    return loss_c(cfg, pos, x, seg, w, nbr, go)
                return loss_c(cfg, pos, h, seg, dict(w, **{name: x}), nbr, go)
            fd = (at(eps) - at(-eps)) / (2 * eps)
            assert abs(fd - g[name].reshape(-1)[f]) <= 1e-6 * max(1.0, abs(fd)), (name, f, fd, g[name].reshape(-1)[f])


def test_position_gradient_sums_to_zero_and_carries_no_torque():
    """Translation invariance: the forces sum to zero per segment.  (Rotation invariance holds only for a scalar
    loss; sum(out * fixed) is not one, so no torque statement is made for it - an invariant loss is used instead.)"""
    cfg, pos, seg, h, w, nbr, go = case(8, L=2, C=8, H=2)
    _, g = G.attn_backward(cfg, pos, h, w, nbr, go, wrt=("pos",))
    for s in range(len(seg) - 1):
        np.testing.assert_allclose(g["pos"][seg[s]:seg[s + 1]].sum(0), 0.0, atol=1e-10)
    # an invariant loss: only the l = 0 block of the output of l = 0 features -> zero net torque
    h0 = h.copy()
    h0[:, 1:] = 0.0
    go0 = np.zeros_like(go)
    go0[:, 0] = go[:, 0]
    _, g0 = G.attn_backward(cfg, pos, h0, w, nbr, go0, wrt=("pos",))
    torque = np.cross(pos, g0["pos"]).sum(0)
    np.testing.assert_allclose(torque, 0.0, atol=1e-9)


def test_periodic_translations_enter_the_pair_vectors():
    from test_oracle_periodic import grid_case
    cfg, pos, seg, h, w, box = grid_case(3, n=40)
    nbr = O.neighbor_list_periodic(pos, seg, cfg["cutoff"], box)
    tr = O.edge_translations(seg, box, nbr[0], nbr[2])
    go = np.random.default_rng(1).normal(size=h.shape)
    folded = O.wrap_positions(pos, seg, box).astype(np.float64)
    out, g = G.attn_backward(cfg, folded, h, w, (nbr[0], nbr[1]), go, translation=tr)
    ref = O.attn_forward(cfg, pos, h, seg, w, box=box, nbr=nbr)
    np.testing.assert_allclose(out, ref, atol=1e-12)
    np.testing.assert_allclose(g["pos"].sum(0), 0.0, atol=1e-10)


def test_gradients_with_respect_to_q_k_v_chain_to_the_gradient_with_respect_to_h():
    """dL/dh assembled by hand from dL/dq, dL/dk, dL/dv through the l-wise maps equals autograd's dL/dh."""
    cfg, pos, seg, h, w, nbr, go = case(4, L=2, C=4, H=2, per_seg=9)
    _, g = G.attn_backward(cfg, pos, h, w, nbr, go, wrt=("q", "k", "v"))
    _, gh = G.attn_backward(cfg, pos, h, w, nbr, go, wrt=("h",))
    L = cfg["L"]
    dh = np.zeros_like(h)
    for l in range(L + 1):
        blk = slice(l * l, (l + 1) ** 2)
        x = h[:, blk]                                               # [N][2l+1][C]
        for W1, W2, gq in ((w["WQ1"][l], w["WQ2"][l], g["q"][:, l]), (w["WK1"][l], w["WK2"][l], g["k"][:, l])):
            a1, a2 = x @ W1.T, x @ W2.T
            dh[:, blk] += (gq[:, None, :] * a2) @ W1 + (gq[:, None, :] * a1) @ W2
        dh[:, blk] += g["v"][:, blk] @ w["WV"][l]
    assert np.abs(gh["h"]).max() > 1e-3
    np.testing.assert_allclose(dh, gh["h"], atol=1e-12)
