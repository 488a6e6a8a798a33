"""GPU parity of e2f_attn_backward against the gradient reference (the operator's definition under float64 autograd,
oracle/grad.py), element by element, through the C-ABI: gradients with respect to positions, to q, k, v and to h."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2601_16622_amd import binding as B
    B.load()   # fails loudly if the HIP library was not built
    return torch


def rel_l2(a, b):
    nb = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / nb) if nb > 0 else float(np.linalg.norm(a - b))


def run_backward(torch, wl, seed=0):
    import oracle as O
    from oracle import grad as G
    from paper_2601_16622_amd import binding as B
    cfg = wl["cfg"]
    ocfg = {k: cfg[k] for k in ("L", "C", "H", "B", "lf", "cutoff")}
    box = wl.get("box")
    if box is None:
        nbr = O.neighbor_list(wl["pos"], wl["seg"], np.float32(cfg["cutoff"]))
        pos64, tr = wl["pos"].astype(np.float64), None
    else:
        full = O.neighbor_list_periodic(wl["pos"], wl["seg"], np.float32(cfg["cutoff"]), box)
        nbr = (full[0], full[1])
        tr = O.edge_translations(wl["seg"], box, full[0], full[2])
        pos64 = O.wrap_positions(wl["pos"], wl["seg"], box).astype(np.float64)
        assert full[2].any()
    go = np.random.default_rng(seed).normal(size=wl["h"].shape).astype(np.float32)
    ref_out, ref = G.attn_backward(ocfg, pos64, wl["h"], wl["weights"], nbr, go, translation=tr,
                                   wrt=("pos", "q", "k", "v"))
    _, ref_h = G.attn_backward(ocfg, pos64, wl["h"], wl["weights"], nbr, go, translation=tr,
                               wrt=("h", "Wb", "w_path", "WQ1", "WQ2", "WK1", "WK2", "WV"))
    ref.update(ref_h)
    ref["W"] = np.stack([ref[k] for k in ("WQ1", "WQ2", "WK1", "WK2", "WV")])
    P = B.Problem(wl)
    try:
        P.build_cells()
        P.forward()
        torch.cuda.synchronize()
        assert rel_l2(P.out.cpu().numpy().astype(np.float64), ref_out) <= TOL[cfg["dtype"]]
        g = torch.from_numpy(go).to(P.device)
        got = [x.cpu().numpy().astype(np.float64) for x in P.backward(g, with_weights=True)]
        torch.cuda.synchronize()
        # The pair work runs in tile form where the forward pass does (with the gradients of Wb and w_path only up to
        # 8 radial functions; beyond that asking for them selects the per-atom kernels: other kernels, other rounding,
        # each checked against the reference on its own); elsewhere it is the same kernels and the same numbers.
        plain = P.backward(g)
        torch.cuda.synchronize()
        same_kernels = not (cfg["dtype"] == "bf16" and cfg["C"] // cfg["H"] == 16 and cfg["B"] <= 16 and cfg["C"] in (32, 64, 128, 256))
        errs = {}
        for name, x, y in zip(("pos", "q", "k", "v", "h"), plain, P.backward(g, with_weights=True)):
            if same_kernels:
                assert torch.equal(x, y)
            x = x.cpu().numpy().astype(np.float64)
            assert np.isfinite(x).all(), name
            errs["plain " + name] = rel_l2(x, ref[name])
            assert errs["plain " + name] <= TOL[cfg["dtype"]], (name, errs)
        for name, arr in zip(("pos", "q", "k", "v", "h", "Wb", "w_path", "W"), got):
            assert np.isfinite(arr).all(), name
            assert np.abs(ref[name]).max() > 1e-6, name
            errs[name] = rel_l2(arr, ref[name])
            assert errs[name] <= TOL[cfg["dtype"]], (name, errs)
        print(errs)
        plain_pos = plain[0].cpu().numpy().astype(np.float64)
        # translation invariance: the position gradients of every segment sum to zero.  The per-atom kernels form a
        # pair's term with the same arithmetic on both of its atoms; the tile kernels round the two sides' operands
        # differently (G^T g against v, g against G v, in bf16), so there the sum is zero to the tolerance only.
        for s in range(len(wl["seg"]) - 1):
            seg = slice(wl["seg"][s], wl["seg"][s + 1])
            for gp, exact in ((got[0][seg], same_kernels or cfg["B"] > 8), (plain_pos[seg], same_kernels)):
                bound = 1e-3 * max(1.0, np.abs(gp).max()) if exact else TOL[cfg["dtype"]] * max(1.0, np.linalg.norm(gp))
                assert np.abs(gp.sum(0)).max() <= bound
        return errs
    finally:
        P.close()


def custom(seed, sizes, L, C, H, B, dtype, cutoff, side):
    from paper_2601_16622_amd import workloads as W
    rng = np.random.default_rng(seed)
    cfg = dict(L=L, C=C, H=H, B=B, lf=1, cutoff=cutoff, dtype=dtype)
    pos = [W.dart_throw_box(rng, n, side, origin=rng.uniform(-5, 5, 3)) for n in sizes]
    return W._pack(cfg, pos, rng, elements=False)


@pytest.mark.parametrize("L,C,H", [(1, 16, 2), (2, 32, 2), (3, 64, 1)])
def test_backward_fp32(torch_cuda, L, C, H):
    """Several segments, a single-atom segment (no neighbours: zero gradients), head widths 8, 16 and 64."""
    wl = custom(10 + L, (150, 1, 90), L, C, H, 6, "f32", 3.5, 9.0)
    run_backward(torch_cuda, wl)


def test_backward_bf16_at_the_benchmark_shape(torch_cuda):
    """L = 4, C = 128, 8 heads, bf16 features; more neighbours than one batch of the list holds."""
    wl = custom(20, (260,), 4, 128, 8, 8, "bf16", 6.0, 10.0)
    import oracle as O
    off, _ = O.neighbor_list(wl["pos"], wl["seg"], np.float32(6.0))
    assert np.diff(off).max() > 128
    run_backward(torch_cuda, wl)


def test_backward_periodic(torch_cuda):
    from paper_2601_16622_amd import workloads as W
    wl = W.periodic_boxes((220, 120), seed=5, L=2, C=32, H=2, B=6, cutoff=4.0, dtype="f32")
    run_backward(torch_cuda, wl)


def test_backward_tile_form_with_12_radial_functions(torch_cuda):
    """The tile kernels' instances for more than 8 radial basis functions (the bias polynomial and its derivative)."""
    wl = custom(21, (230, 40), 3, 64, 4, 12, "bf16", 4.5, 11.0)
    run_backward(torch_cuda, wl)


def test_backward_tile_form_256_channels(torch_cuda):
    """A channel count the tile-layout projection is not built for: plain projection, relayout, tile kernels; the chain
    rule through the projections on the vector-ALU kernel."""
    wl = custom(22, (200, 60), 2, 256, 16, 8, "bf16", 4.5, 11.0)
    run_backward(torch_cuda, wl)


def test_backward_tile_form_periodic(torch_cuda):
    """bf16 features and heads of 16 channels in periodic boxes: the tile kernels of the backward pass with candidate
    lists that include images (a source sees its targets at the opposite images)."""
    from paper_2601_16622_amd import workloads as W
    wl = W.periodic_boxes((300, 150), seed=6, L=2, C=32, H=2, B=8, cutoff=4.0, dtype="bf16")
    run_backward(torch_cuda, wl)


def test_backward_tile_form_with_crowded_tiles(torch_cuda):
    """1500 atoms in a 6 A cube inside a sparse shell, and a sparse cluster apart: the dense tiles keep more slot groups
    than a tile's candidate list holds (192 entries; the same recipe as the forward pass's test of long lists) and
    are left to the per-atom kernels, which read the tile layouts and exchange the softmax statistics with the tile
    kernels of the sparse tiles around them."""
    from paper_2601_16622_amd import workloads as W
    rng = np.random.default_rng(12)
    cfg = dict(L=1, C=32, H=2, B=8, lf=1, cutoff=4.0, dtype="bf16")
    mixed = np.concatenate([W.dart_throw_box(rng, 1500, 6.0, min_sep=0.3, origin=(5.0, 5.0, 5.0)),
                            W.dart_throw_box(rng, 250, 16.0, min_sep=1.5)])
    sparse = W.dart_throw_box(rng, 200, 14.0, origin=(40.0, 0.0, 0.0))
    wl = W._pack(cfg, [mixed, sparse], rng, elements=False)
    import oracle as O
    offs, _ = O.neighbor_list(wl["pos"], wl["seg"], np.float32(4.0))
    deg = np.diff(offs)
    assert deg[:1500].max() > 4 * 256 and deg[1750:].max() < 100
    assert ((deg[1500:1750] > 100) & (deg[1500:1750] < 600)).any()   # shell atoms that see part of the core
    run_backward(torch_cuda, wl)


def test_backward_after_forward_reuses_the_workspace(torch_cuda):
    """e2f_attn_backward_after_forward reads the projections and candidate lists that the forward pass left in the
    workspace: the same kernels on the same numbers as the stand-alone call, so every gradient agrees bit for bit
    (tile form: bf16 at the benchmark's shape, open and periodic cells, a crowded core); a configuration whose backward
    pass has no tile form takes the stand-alone path and agrees as well."""
    from paper_2601_16622_amd import binding as B, workloads as W
    rng = np.random.default_rng(5)
    crowded = np.concatenate([W.dart_throw_box(rng, 700, 5.0, min_sep=0.3, origin=(4.0, 4.0, 4.0)),
                              W.dart_throw_box(rng, 150, 13.0, min_sep=1.5)])
    cases = [W.box(1500, 2), W.periodic_boxes((700,), 3), W.box(300, 4, dtype="f32", C=64, H=4),
             W._pack(dict(L=2, C=64, H=4, B=8, lf=1, cutoff=4.0, dtype="bf16"), [crowded], rng, elements=False)]
    for wl in cases:
        P = B.Problem(wl)
        try:
            P.build_cells()
            g = torch_cuda.randn(P.out.shape, generator=torch_cuda.Generator().manual_seed(1)).to(P.device)
            P.forward()
            alone = [x.clone() for x in P.backward(g)]
            for x in P.backward(g): x.fill_(float("nan"))
            P.forward(for_backward=True)
            for with_weights in (False, True):
                saved = P.backward(g, after_forward=True, with_weights=with_weights)
                torch_cuda.cuda.synchronize()
                for a, b in zip(alone, saved[:5]):
                    assert torch_cuda.equal(a, b)
            ref_w = P.backward(g, with_weights=True)
            torch_cuda.cuda.synchronize()
            for a, b in zip(ref_w[5:], saved[5:]):
                assert torch_cuda.equal(a, b)
        finally:
            P.close()


def test_backward_rejects_what_it_does_not_cover(torch_cuda):
    from paper_2601_16622_amd import binding as B
    wl = custom(30, (60,), 2, 32, 2, 4, "f32", 3.5, 7.0)
    wl["cfg"]["lf"] = 2
    P = B.Problem(wl)
    try:
        P.build_cells()
        P.forward()
        with pytest.raises(B.E2fError) as e:
            P.backward(torch_cuda.zeros_like(P.out))
        assert e.value.code == 2
    finally:
        P.close()


def test_backward_scaling_point_sampled(torch_cuda):
    """The 10 000-atom box the benchmark times, bf16, same launch configuration: dL/dpos and dL/dh of 120 atoms (a
    compact cluster that reaches a face of the box, so surface atoms are among them) against the gradient reference.
    The gradient with respect to atom a involves only the outputs of a and of its neighbours, so the reference runs
    on those targets (with their complete neighbourhoods) alone, all 120 atoms in one differentiation."""
    import oracle as O
    from oracle import grad as G
    from paper_2601_16622_amd import binding as B
    from paper_2601_16622_amd import workloads as W
    wl = W.scaling_point(0)
    cfg = wl["cfg"]
    ocfg = {k: cfg[k] for k in ("L", "C", "H", "B", "lf", "cutoff")}
    N = wl["pos"].shape[0]
    off, idx = O.neighbor_list(wl["pos"], wl["seg"], np.float32(cfg["cutoff"]), use_cells=True)
    go = np.random.default_rng(7).normal(size=wl["h"].shape).astype(np.float32)
    P = B.Problem(wl)
    try:
        P.build_cells()
        P.forward()
        gp, _, _, _, gh = P.backward(torch_cuda.from_numpy(go).to(P.device))
        torch_cuda.cuda.synchronize()
        gp, gh = gp.cpu().numpy().astype(np.float64), gh.cpu().numpy().astype(np.float64)
    finally:
        P.close()
    assert np.isfinite(gp).all() and np.isfinite(gh).all()
    assert np.abs(gp.sum(0)).max() <= 1e-3 * np.abs(gp).max() * np.sqrt(N)   # translation invariance
    pos = wl["pos"].astype(np.float64)
    centre = np.array([pos[:, 0].min() + 3.0, pos[:, 1].mean(), pos[:, 2].mean()])   # three angstrom inside a face
    picks = np.argsort(((pos - centre) ** 2).sum(1))[:120]
    assert (pos[picks, 0] < pos[:, 0].min() + 0.5).any() and np.diff(off)[picks].min() < 60 < np.diff(off)[picks].max()
    targets = np.unique(np.concatenate([picks] + [idx[off[a]:off[a + 1]] for a in picks]))
    atoms = np.unique(np.concatenate([targets] + [idx[off[i]:off[i + 1]] for i in targets]))
    local = -np.ones(N, dtype=np.int64)
    local[atoms] = np.arange(len(atoms))
    rows = [np.zeros(0, dtype=np.int32)] * len(atoms)
    for i in targets:
        rows[local[i]] = local[idx[off[i]:off[i + 1]]].astype(np.int32)
    sub_off = np.zeros(len(atoms) + 1, dtype=np.int64)
    sub_off[1:] = np.cumsum([len(r) for r in rows])
    sub_go = np.zeros((len(atoms),) + go.shape[1:], dtype=np.float64)
    sub_go[local[targets]] = go[targets]
    _, g = G.attn_backward(ocfg, pos[atoms], wl["h"][atoms], wl["weights"], (sub_off, np.concatenate(rows)), sub_go,
                           wrt=("pos", "h"))
    ref_p, ref_h = g["pos"][local[picks]], g["h"][local[picks]]
    assert rel_l2(gp[picks], ref_p) <= TOL["bf16"]
    assert rel_l2(gh[picks], ref_h) <= TOL["bf16"]
    # no single atom hides in the norm over all of them
    for got, ref in ((gp[picks], ref_p), (gh[picks], ref_h)):
        d = np.linalg.norm((got - ref).reshape(len(picks), -1), axis=1)
        r = np.linalg.norm(ref.reshape(len(picks), -1), axis=1)
        assert (d <= 5 * TOL["bf16"] * np.maximum(r, 0.05 * r.mean())).all(), float((d / r).max())
