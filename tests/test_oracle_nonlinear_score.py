"""Pins for the oracle's logit with the non-linear pair feature (App. "Role of Non-linearity", Eqs. app-nonlin-fea and
app-nonlin-alpha, in the reading stated at e2fo_attn_forward): symmetries, the scalar case written with dense torch
ops, a collinear configuration whose harmonics are known in closed form, and what switching the feature off gives."""
import numpy as np

import oracle as O
from test_oracle_operator import Ry, Rz, rotate_features, small_case

RNG = np.random.default_rng(99)


def silu(x):
    return x / (1.0 + np.exp(-x))


def test_rotation_equivariance():
    """The feature is built from invariants (degree-wise inner products with the harmonics of the pair direction), so
    the operator stays equivariant; a harmonic in the wrong basis or order would break this."""
    for lf in (1, 2):
        cfg, pos, seg, h, w = small_case(21, lf=lf)
        a, b, g = RNG.uniform(-3, 3, size=3)
        R = Rz(a) @ Ry(b) @ Rz(g)
        out = O.attn_forward(cfg, pos, h, seg, w, score_mode="nonlinear")
        out_rot = O.attn_forward(cfg, pos @ R.T, rotate_features(h, cfg["L"], a, b, g), seg, w, score_mode="nonlinear")
        assert np.abs(out).max() > 0.1
        np.testing.assert_allclose(out_rot, rotate_features(out, cfg["L"], a, b, g), atol=1e-10)


def test_the_feature_changes_the_result_and_keeps_the_symmetries():
    cfg, pos, seg, h, w = small_case(22)
    plain = O.attn_forward(cfg, pos, h, seg, w)
    out = O.attn_forward(cfg, pos, h, seg, w, score_mode="nonlinear")
    assert np.abs(out - plain).max() > 1e-3
    np.testing.assert_allclose(O.attn_forward(cfg, pos + np.array([0.3, -1.1, 2.0]), h, seg, w, score_mode="nonlinear"),
                               out, atol=1e-10)
    np.testing.assert_allclose(O.attn_forward(cfg, pos, h, seg, w, score_mode="nonlinear", softmax_mode="streaming",
                                              message_mode="eaas"), out, atol=1e-11)
    perm = np.concatenate([RNG.permutation(14), 14 + RNG.permutation(14)])
    np.testing.assert_allclose(O.attn_forward(cfg, pos[perm], h[perm], seg, w, score_mode="nonlinear"), out[perm],
                               atol=1e-11)


def test_scalar_case_with_dense_torch_ops():
    """L = 0, l_f = 0: Y^(0) = 1, so a = W_Q1 h_i and b = W_V h_j and the logit is
    tau sum_c q_i[c] k_j[c] (silu(a_i[c]) + silu(b_j[c])) + bias: two dense matrix products per head."""
    import torch
    from paper_2601_16622_amd import workloads as W
    rng = np.random.default_rng(12)
    N, C, H, B, rc = 36, 12, 3, 5, 2.5
    pos = W.dart_throw_box(rng, N, 6.0).astype(np.float64)
    seg = np.array([0, 20, N], dtype=np.int32)
    cfg = dict(L=0, C=C, H=H, B=B, lf=0, cutoff=rc)
    h = rng.normal(size=(N, 1, C))
    w = {k: rng.normal(size=(1, C, C)) / np.sqrt(C) for k in ("WQ1", "WQ2", "WK1", "WK2", "WV")}
    w["Wb"] = rng.normal(size=(H, B))
    w["w_path"] = np.array([[0.9]])
    out = O.attn_forward(cfg, pos, h, seg, w, score_mode="nonlinear")

    x = torch.tensor(h[:, 0])
    T = {k: torch.tensor(v[0]) for k, v in w.items() if k.startswith("W") and k != "Wb"}
    q1 = x @ T["WQ1"].T
    q = q1 * (x @ T["WQ2"].T)
    k = (x @ T["WK1"].T) * (x @ T["WK2"].T)
    v = x @ T["WV"].T
    Ch = C // H
    p = torch.tensor(pos)
    d = torch.cdist(p, p)
    seg_of = torch.tensor(np.searchsorted(seg, np.arange(N), side="right"))
    mask = (d < rc) & (d > 0) & (seg_of[:, None] == seg_of[None, :])
    mu = torch.arange(B, dtype=torch.float64) * rc / (B - 1)
    g = torch.exp(-0.5 * (B - 1) ** 2 / rc ** 2 * (d[..., None] - mu) ** 2)
    bias = torch.einsum("ijb,hb->hij", g, torch.tensor(w["Wb"]))
    heads = lambda t: t.reshape(N, H, Ch).permute(1, 0, 2)
    qh, kh, vh = heads(q), heads(k), heads(v)
    fa, fb = heads(torch.nn.functional.silu(q1)), heads(torch.nn.functional.silu(v))
    s = ((qh * fa) @ kh.transpose(1, 2) + qh @ (kh * fb).transpose(1, 2)) / np.sqrt(Ch) + bias
    s = s.masked_fill(~mask, float("-inf"))
    a = torch.nan_to_num(torch.softmax(s, dim=-1), nan=0.0) * (0.5 * (1 + torch.cos(np.pi * d / rc)))
    ref = 0.9 * (a @ vh).permute(1, 0, 2).reshape(N, C)
    np.testing.assert_allclose(out[:, 0], ref.numpy(), atol=1e-12)


def test_three_atoms_on_the_z_axis():
    """Target at the origin, neighbours at +z and -z: Y^(l)_m(+-z) = (+-1)^l [m = 0] (components ordered m = -l..l, so
    m = 0 is the middle one).  The two logits follow from the m = 0 components alone; the output is checked through
    the ratio of the two softmax weights, recovered from the l_f = 0 message (which is w_path[l][l] v_j)."""
    rng = np.random.default_rng(5)
    L, C, H, B, rc = 2, 4, 2, 3, 3.0
    n, Ch = (L + 1) ** 2, C // H
    pos = np.array([[0, 0, 0], [0, 0, 1.2], [0, 0, -1.7]], dtype=np.float64)
    seg = np.array([0, 3], dtype=np.int32)
    cfg = dict(L=L, C=C, H=H, B=B, lf=0, cutoff=rc)
    h = rng.normal(size=(3, n, C))
    w = {k: rng.normal(size=(L + 1, C, C)) / np.sqrt(C) for k in ("WQ1", "WQ2", "WK1", "WK2", "WV")}
    w["Wb"] = rng.normal(size=(H, B))
    w["w_path"] = np.diag(rng.uniform(0.5, 1.5, size=L + 1))
    out = O.attn_forward(cfg, pos, h, seg, w, targets=np.array([0], dtype=np.int32), score_mode="nonlinear")[0]

    def proj(Wm, x):   # l-wise map of one atom: [n][C]
        return np.concatenate([x[l * l:(l + 1) ** 2] @ Wm[l].T for l in range(L + 1)])

    def inv(a, b):
        return np.stack([(a[l * l:(l + 1) ** 2] * b[l * l:(l + 1) ** 2]).sum(0) for l in range(L + 1)])

    q1 = proj(w["WQ1"], h[0])
    q = inv(q1, proj(w["WQ2"], h[0]))
    mid = [l * l + l for l in range(L + 1)]
    ref = np.zeros((n, C))
    logits, gates, vals = [], [], []
    for j, sign in ((1, 1.0), (2, -1.0)):
        k = inv(proj(w["WK1"], h[j]), proj(w["WK2"], h[j]))
        v = proj(w["WV"], h[j])
        par = np.array([sign ** l for l in range(L + 1)])[:, None]
        fea = silu(par * q1[mid]) + silu(par * v[mid])                      # [L+1][C]
        d = abs(pos[j, 2])
        mu = np.arange(B) * rc / (B - 1)
        bias = w["Wb"] @ np.exp(-0.5 * (B - 1) ** 2 / rc ** 2 * (d - mu) ** 2)
        s = (q * k * fea).reshape(L + 1, H, Ch).sum((0, 2)) / np.sqrt((L + 1) * Ch) + bias
        logits.append(s)
        gates.append(0.5 * (1 + np.cos(np.pi * d / rc)))
        vals.append(v)
    logits = np.array(logits)
    p = np.exp(logits - logits.max(0))
    p /= p.sum(0)
    for e in range(2):
        for l in range(L + 1):
            ref[l * l:(l + 1) ** 2] += (w["w_path"][l, l] * gates[e] * np.repeat(p[e], Ch))[None, :] * vals[e][l * l:(l + 1) ** 2]
    np.testing.assert_allclose(out, ref, atol=1e-12)


def test_vanishing_higher_degrees_leave_the_scalar_feature():
    """With all l > 0 features zero the invariants a, b of l > 0 vanish, silu(0) = 0, and q, k of l > 0 vanish too: the
    result must equal the L = 0 operator on the scalar block (embedded weights)."""
    cfg, pos, seg, h, w = small_case(23, L=2, lf=0)
    h[:, 1:] = 0.0
    out = O.attn_forward(cfg, pos, h, seg, w, score_mode="nonlinear")
    cfg0 = dict(cfg, L=0)
    w0 = {k: w[k][:1] for k in ("WQ1", "WQ2", "WK1", "WK2", "WV")}
    w0["Wb"] = w["Wb"]
    w0["w_path"] = w["w_path"][:1, :1]
    # the logit scale 1/sqrt(d_k) differs between L = 2 and L = 0 (d_k = (L+1) C_h): fold the ratio into W_Q2
    w0["WQ2"] = w0["WQ2"] / np.sqrt(3.0)
    out0 = O.attn_forward(cfg0, pos, h[:, :1], seg, w0, score_mode="nonlinear")
    np.testing.assert_allclose(out[:, :1], out0, atol=1e-12)
    assert np.abs(out[:, 1:]).max() == 0.0
