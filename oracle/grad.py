"""Gradients of the operator: test infrastructure, like the rest of this package.

The paper gives only the forward pass (Algorithm 1 is headed "Forward Pass"; conservative forces F = -dE/dpos and
training need its derivative).  The reference here is reverse-mode differentiation, by torch.autograd in float64, of
the operator's definition written out in plain tensor operations for the degree-1 filter:

    q, k  = invariants of the l-wise projections (Eq. qk),  v = W_V h
    s     = q.k / sqrt(d_k) + b_h(|r|),  alpha = softmax_j(s) phi(|r|)          (Eq. attn, gate outside the softmax)
    out_i = sum_j alpha_ij sum_li w_path[li][lo] CG^{lo}_{li,1} (v_j^{li}, R^1(r_ij))   (the dense definition)

The forward value of this route is pinned to the C oracle, its gradients to central differences of the C oracle
(tests/test_oracle_grad.py).  Pair vectors are r_ij = (pos_j + translation_e) - pos_i on the edge list handed in, so
the derivative holds the neighbour sets fixed, as any derivative of a cutoff model does.
"""
import numpy as np
import torch

from . import cg_real, solid_harmonics


def _edges(offsets, idx):
    offsets = np.asarray(offsets, dtype=np.int64)
    tgt = np.repeat(np.arange(len(offsets) - 1), np.diff(offsets))
    return torch.from_numpy(tgt.astype(np.int64)), torch.from_numpy(np.asarray(idx, dtype=np.int64))


def project_qkv(cfg, h, weights):
    """q, k [N][L+1][C] (the invariants of Eq. qk, unscaled) and v [N][n][C] from the l-wise projections."""
    L = cfg["L"]

    def project(W):   # [L+1][C][C] (out, in) applied l-wise
        blocks = [torch.einsum("oc,nmc->nmo", W[l], h[:, l * l:(l + 1) ** 2]) for l in range(L + 1)]
        return torch.cat(blocks, dim=1)

    def invariant(a, b):   # sum over m inside every degree: [N][L+1][C]
        return torch.stack([(a[:, l * l:(l + 1) ** 2] * b[:, l * l:(l + 1) ** 2]).sum(1) for l in range(L + 1)], 1)

    q = invariant(project(weights["WQ1"]), project(weights["WQ2"]))
    k = invariant(project(weights["WK1"]), project(weights["WK2"]))
    return q, k, project(weights["WV"])


def forward_torch(cfg, pos, h, weights, nbr, translation=None, qkv=None):
    """The operator on torch float64 tensors (pos [N][3], h [N][n][C], weights as in oracle.attn_forward; any of them
    may require grad).  nbr = (offsets, idx) CSR lists, translation = None or [E][3] lattice translations.
    qkv: None, or (q, k, v) tensors to use in place of the projections of h (to differentiate with respect to them).
    Returns out [N][n][C]."""
    L, C, H, B, lf = cfg["L"], cfg["C"], cfg["H"], cfg["B"], cfg["lf"]
    if lf != 1:
        raise ValueError("the differentiable route is written for the degree-1 filter")
    rc = float(np.float32(cfg["cutoff"]))
    n, Ch = (L + 1) ** 2, C // H
    N = pos.shape[0]
    ti, sj = _edges(*nbr)
    E = ti.shape[0]
    f64 = torch.float64

    q, k, v = project_qkv(cfg, h, weights) if qkv is None else qkv
    out = torch.zeros((N, n, C), dtype=f64)
    if E == 0:
        return out + 0.0 * (q.sum() + k.sum() + v.sum())

    r = pos[sj] - pos[ti]
    if translation is not None:
        r = r + torch.as_tensor(np.asarray(translation, dtype=np.float64))
    d = torch.sqrt((r * r).sum(1))
    # radial bias and gate
    if B > 1:
        mu = torch.arange(B, dtype=f64) * (rc / (B - 1))
        gamma = (B - 1) ** 2 / (2.0 * rc * rc)
    else:
        mu = torch.zeros(1, dtype=f64)
        gamma = 1.0 / (2.0 * rc * rc)
    g = torch.exp(-gamma * (d[:, None] - mu[None, :]) ** 2)            # [E][B]
    bias = g @ weights["Wb"].T                                            # [E][H]
    gate = 0.5 * (1.0 + torch.cos(np.pi * d / rc))
    # logits per head
    tau = 1.0 / np.sqrt((L + 1) * Ch)
    qh = q.reshape(N, L + 1, H, Ch)
    kh = k.reshape(N, L + 1, H, Ch)
    s = tau * (qh[ti] * kh[sj]).sum((1, 3)) + bias                        # [E][H]
    # softmax over the neighbours of every target
    smax = torch.full((N, H), -np.inf, dtype=f64).scatter_reduce(0, ti[:, None].expand(E, H), s.detach(), "amax")
    p = torch.exp(s - smax[ti])
    z = torch.zeros((N, H), dtype=f64).index_add(0, ti, p)
    alpha = p / z[ti] * gate[:, None]                                     # [E][H]
    # the degree-1 solid harmonic is linear in r: R^1(r) = A r, A read off the C oracle on the unit vectors
    A = torch.from_numpy(np.stack([solid_harmonics(1, e) for e in np.eye(3)], axis=1))   # [3 (m)][3 (axis)]
    R1 = r @ A.T                                                          # [E][3]
    vj = v[sj]                                                            # [E][n][C]
    blocks = []
    for lo in range(L + 1):
        acc = torch.zeros((E, 2 * lo + 1, C), dtype=f64)
        for li in range(L + 1):
            if lo < abs(li - 1) or lo > li + 1:
                continue
            cg = torch.from_numpy(cg_real(li, 1, lo).reshape(2 * lo + 1, 2 * li + 1, 3))
            acc = acc + weights["w_path"][li, lo] * torch.einsum("oif,eic,ef->eoc", cg, vj[:, li * li:(li + 1) ** 2], R1)
        blocks.append(acc)
    msg = torch.cat(blocks, dim=1)                                        # [E][n][C]
    a_c = alpha.repeat_interleave(Ch, dim=1)                              # [E][C]: head of every channel
    return out.index_add(0, ti, msg * a_c[:, None, :])


def attn_backward(cfg, pos, h, weights, nbr, grad_out, translation=None, wrt=("pos", "h")):
    """Gradients of sum(out * grad_out) with respect to the named inputs: "pos", "h", a weight name, or "q", "k",
    "v" (the projections of h taken as independent variables; not together with "h" or projection weights).
    Returns (out, {name: gradient}) as float64 numpy arrays."""
    tp = torch.tensor(np.asarray(pos, dtype=np.float64), requires_grad="pos" in wrt)
    th = torch.tensor(np.asarray(h, dtype=np.float64), requires_grad="h" in wrt)
    tw = {kk: torch.tensor(np.asarray(vv, dtype=np.float64), requires_grad=kk in wrt) for kk, vv in weights.items()}
    qkv = None
    if any(name in wrt for name in ("q", "k", "v")):
        with torch.no_grad():
            qkv = project_qkv(cfg, th, tw)
        qkv = tuple(t.clone().requires_grad_(name in wrt) for t, name in zip(qkv, ("q", "k", "v")))
    out = forward_torch(cfg, tp, th, tw, nbr, translation, qkv)
    loss = (out * torch.as_tensor(np.asarray(grad_out, dtype=np.float64))).sum()
    if wrt:
        loss.backward()
    grads = {}
    for name in wrt:
        t = (tp if name == "pos" else th if name == "h" else qkv["qkv".index(name)] if name in ("q", "k", "v")
             else tw[name])
        grads[name] = (t.grad if t.grad is not None else torch.zeros_like(t)).numpy()
    return out.detach().numpy(), grads
