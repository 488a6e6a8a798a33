"""GPU parity under periodic boundaries: e2f_build_cells_periodic, then the neighbour sets, the fused forward pass and
its capped form against the oracle's periodic route, element by element, through the C-ABI."""
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


def oracle_cfg(wl):
    return {k: wl["cfg"][k] for k in ("L", "C", "H", "B", "lf", "cutoff")}


def run_periodic(torch, wl, targets=None, cap=None, attention="auto"):
    """Neighbour sets exactly, forward within the tolerance of the dtype; returns the relative L2 error."""
    import oracle as O
    from paper_2601_16622_amd import binding as B
    cfg = wl["cfg"]
    P = B.Problem(wl, attention=attention)
    try:
        P.build_cells()
        deg, offs, idx = P.neighbors()
        nbr = O.neighbor_list_periodic(wl["pos"], wl["seg"], np.float32(cfg["cutoff"]), wl["box"])
        assert np.array_equal(offs, nbr[0]), "neighbour counts differ"
        assert np.array_equal(idx, nbr[1]), "neighbour sets differ"
        assert nbr[2].any(), "no pair crosses a face: the case does not test images"
        use = nbr
        if cap is not None:
            folded = O.wrap_positions(wl["pos"], wl["seg"], wl["box"])
            tr = O.edge_translations(wl["seg"], wl["box"], nbr[0], nbr[2])
            c_off, c_idx, kept = O.cap_neighbors(folded, nbr[0], nbr[1], cap, translation=tr)
            assert (np.diff(nbr[0]) > cap).any()
            use = (c_off, c_idx, nbr[2][kept])
        ref = O.attn_forward(oracle_cfg(wl), wl["pos"], wl["h"], wl["seg"], wl["weights"], targets=targets, nbr=use,
                             box=wl["box"], message_mode="eaas")
        sel = slice(None) if targets is None else targets
        P.out.fill_(float("nan"))
        if cap is None:
            P.forward()
        else:
            P.forward_capped(cap)
        torch.cuda.synchronize()
        got = P.out.cpu().numpy().astype(np.float64)
        assert np.isfinite(got).all()
        assert np.abs(ref).max() > 1e-3
        err = rel_l2(got[sel], ref)
        assert err <= TOL[cfg["dtype"]], f"rel L2 {err}"
        for l in range(cfg["L"] + 1):
            blk = slice(l * l, (l + 1) ** 2)
            if np.linalg.norm(ref[:, blk]) > 0:
                assert rel_l2(got[sel][:, blk], ref[:, blk]) <= TOL[cfg["dtype"]]
        return err
    finally:
        P.close()


@pytest.mark.parametrize("kernel", ["tile", "pair", "valu"])
def test_two_periodic_boxes_bf16(torch_cuda, kernel):
    """Two boxes of different size in one batch, coordinates partly outside [0, len), tiles that span faces."""
    from paper_2601_16622_amd import workloads as W
    wl = W.periodic_boxes((700, 420), seed=1, L=2, C=64, H=4, B=8, cutoff=5.0, dtype="bf16")
    run_periodic(torch_cuda, wl, attention=kernel)


def test_periodic_box_at_the_benchmark_shape_sampled(torch_cuda):
    """L = 4, C = 128, 8 heads (the tile kernel at the benchmark's shape), sampled targets."""
    from paper_2601_16622_amd import workloads as W
    wl = W.periodic_boxes((2500,), seed=2)
    tg = np.random.default_rng(5).choice(2500, 150, replace=False).astype(np.int32)
    run_periodic(torch_cuda, wl, targets=tg)


def test_two_periodic_boxes_fp32_tile_kernel(torch_cuda):
    """fp32 features and heads of 16 channels: the fp32 tile kernel over candidate lists with images, L_max = 4."""
    from paper_2601_16622_amd import workloads as W
    wl = W.periodic_boxes((700, 300), seed=8, L=4, C=64, H=4, B=8, cutoff=5.0, dtype="f32")
    run_periodic(torch_cuda, wl, attention="tile")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_periodic_all_degrees_of_the_filter(torch_cuda, dtype):
    """lf = 1 and 2; in bf16 the degree-2 filter runs on the per-pair matrix-core kernel."""
    from paper_2601_16622_amd import workloads as W
    for lf in (1, 2):
        wl = W.periodic_boxes((260, 150, 1), seed=3 + lf, L=2, C=32, H=2, B=6, cutoff=4.0, dtype=dtype)
        wl["cfg"]["lf"] = lf
        run_periodic(torch_cuda, wl)


@pytest.mark.parametrize("open_axes", [(2,), (0, 1)])
def test_slab_and_wire(torch_cuda, open_axes):
    """Mixed boundaries: periodic along some axes, open along the others."""
    from paper_2601_16622_amd import workloads as W
    wl = W.periodic_boxes((500,), seed=7, L=2, C=64, H=4, cutoff=5.0, dtype="bf16", open_axes=open_axes)
    run_periodic(torch_cuda, wl)


def test_periodic_and_open_segments_in_one_batch(torch_cuda):
    """A periodic box next to an open cluster (all three box entries zero) and an empty segment between them."""
    from paper_2601_16622_amd import workloads as W
    wl = W.periodic_boxes((420, 260), seed=11, L=2, C=64, H=4, cutoff=5.0, dtype="bf16")
    wl["seg"] = np.array([0, 420, 420, 680], dtype=np.int32)
    wl["box"] = np.stack([wl["box"][0], np.zeros(3, dtype=np.float32), np.zeros(3, dtype=np.float32)])
    run_periodic(torch_cuda, wl)


def test_full_fcc_crystal(torch_cuda):
    """Every atom of the periodic crystal has the 54 neighbours of the closed form; many exactly equidistant pairs
    and pair vectors along the axes."""
    from paper_2601_16622_amd import binding as B
    from paper_2601_16622_amd import workloads as W
    wl = W.periodic_fcc(5, L=2, C=64, H=4, dtype="bf16")
    run_periodic(torch_cuda, wl)
    P = B.Problem(wl)
    try:
        P.build_cells()
        deg, _, _ = P.neighbors()
        assert (deg == 54).all()
    finally:
        P.close()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_capped_forward_with_images(torch_cuda, dtype):
    from paper_2601_16622_amd import workloads as W
    wl = W.periodic_boxes((600, 300), seed=9, L=2, C=64, H=4, cutoff=5.0, dtype=dtype)
    run_periodic(torch_cuda, wl, cap=14)


def test_neighbor_table_with_images(torch_cuda):
    import oracle as O
    from paper_2601_16622_amd import binding as B
    from paper_2601_16622_amd import workloads as W
    wl = W.periodic_fcc(5, L=1, C=32, H=2, B=4, dtype="f32")
    nbr = O.neighbor_list_periodic(wl["pos"], wl["seg"], 6.0, wl["box"])
    folded = O.wrap_positions(wl["pos"], wl["seg"], wl["box"])
    tr = O.edge_translations(wl["seg"], wl["box"], nbr[0], nbr[2])
    K = 20   # cuts the third shell: only the index tie rule decides
    c_off, c_idx, _ = O.cap_neighbors(folded, nbr[0], nbr[1], K, translation=tr)
    P = B.Problem(wl)
    try:
        P.build_cells()
        table, count = P.neighbor_table(K)
        torch_cuda.cuda.synchronize()
        table, count = table.cpu().numpy(), count.cpu().numpy()
        assert (count == K).all()
        for i in range(P.N):
            assert np.array_equal(np.sort(table[i]), c_idx[c_off[i]:c_off[i + 1]]), i
    finally:
        P.close()


def test_periodic_scaling_box_sampled(torch_cuda):
    """10 000 atoms in one periodic box (the benchmark's system with its faces closed): every neighbour set, and the
    forward pass on sampled targets, in the launch configuration the benchmark times."""
    from paper_2601_16622_amd import workloads as W
    wl = W.by_name("pbox10000", 0)
    tg = np.random.default_rng(3).choice(10_000, 120, replace=False).astype(np.int32)
    run_periodic(torch_cuda, wl, targets=tg)


def test_what_periodic_cells_do_not_support(torch_cuda):
    from paper_2601_16622_amd import binding as B
    from paper_2601_16622_amd import workloads as W
    wl = W.periodic_boxes((300,), seed=4, L=1, C=32, H=2, cutoff=5.0, dtype="bf16")
    P = B.Problem(wl)
    try:
        P.build_cells()
        for call in (P.forward_factorized, P.forward_materialized):
            with pytest.raises(B.E2fError) as e:
                call()
            assert e.value.code == 2
        table, _ = P.neighbor_table(8)
        with pytest.raises(B.E2fError) as e:
            P.forward_table(table)
        assert e.value.code == 2
        # a box below three cell edges along a periodic axis
        P.box = np.array([[3 * 5.0 * 1.00005, 40.0, 0.0]], dtype=np.float32)
        with pytest.raises(B.E2fError) as e:
            P.build_cells()
        assert e.value.code == 2
        P.box = np.array([[np.inf, 40.0, 40.0]], dtype=np.float32)
        with pytest.raises(B.E2fError) as e:
            P.build_cells()
        assert e.value.code == 2
        P.box = np.array([[0.0, -1.0, np.nan]], dtype=np.float32)   # all open: plain cells
        P.cells = None
        P.build_cells()
        P.forward()
        torch_cuda.cuda.synchronize()
        assert torch_cuda.isfinite(P.out).all()
    finally:
        P.close()
