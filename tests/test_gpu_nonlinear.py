"""GPU parity of e2f_attn_forward_nonlinear (the logit with the non-linear pair feature) against the oracle's
score_mode="nonlinear", element by element through the C-ABI: fp32 and bf16 features, every filter degree, open and
periodic cells, the benchmark's shape on sampled targets."""
import numpy as np
import pytest

from test_gpu_parity import TOL, _custom, rel_l2

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2601_16622_amd import binding as B
    B.load()   # fails loudly if the HIP library was not built
    return torch


def run_nonlinear(torch, wl, targets=None):
    import oracle as O
    from paper_2601_16622_amd import binding as B
    cfg = wl["cfg"]
    ocfg = {k: cfg[k] for k in ("L", "C", "H", "B", "lf", "cutoff")}
    box = wl.get("box")
    P = B.Problem(wl)
    try:
        P.build_cells()
        deg, offs, idx = P.neighbors()
        if box is None:
            nbr = O.neighbor_list(wl["pos"], wl["seg"], np.float32(cfg["cutoff"]), use_cells=P.N > 3000)
        else:
            nbr = O.neighbor_list_periodic(wl["pos"], wl["seg"], np.float32(cfg["cutoff"]), box)
        assert np.array_equal(offs, nbr[0]) and np.array_equal(idx, nbr[1]), "neighbour sets differ"
        kw = dict(targets=targets, nbr=nbr, message_mode="eaas", score_mode="nonlinear")
        if box is not None:
            kw["box"] = box
        ref = O.attn_forward(ocfg, wl["pos"], wl["h"], wl["seg"], wl["weights"], **kw)
        plain = O.attn_forward(ocfg, wl["pos"], wl["h"], wl["seg"], wl["weights"], **dict(kw, score_mode="kernel_score"))
        sel = slice(None) if targets is None else targets
        P.out.fill_(float("nan"))
        P.forward_nonlinear()
        torch.cuda.synchronize()
        got = P.out.cpu().numpy().astype(np.float64)
        assert np.isfinite(got).all()
        err = rel_l2(got[sel], ref)
        assert err <= TOL[cfg["dtype"]], f"rel L2 {err}"
        for l in range(cfg["L"] + 1):
            blk = slice(l * l, (l + 1) ** 2)
            if np.linalg.norm(ref[:, blk]) > 0:
                assert rel_l2(got[sel][:, blk], ref[:, blk]) <= TOL[cfg["dtype"]]
        # the feature matters in this case: the plain logit's result is far outside the tolerance
        if ref.shape[0] > 8 and np.linalg.norm(ref) > 0:
            assert rel_l2(plain, ref) > 10 * TOL[cfg["dtype"]]
        return err
    finally:
        P.close()


@pytest.mark.parametrize("kw", [
    dict(N=50, L=0, C=32, H=4, B=4, lf=0, dtype="f32"),        # scalar case: a = W_Q1 h_i, b = W_V h_j
    dict(N=77, L=2, C=64, H=4, B=1, lf=0, dtype="f32"),        # higher degrees in the feature, identity message
    dict(N=90, L=2, C=64, H=4, B=8, lf=1, dtype="f32"),
    dict(N=61, L=3, C=32, H=2, B=8, lf=1, dtype="bf16"),
    dict(N=90, L=4, C=64, H=8, B=16, lf=1, dtype="f32"),
    dict(N=120, L=2, C=16, H=1, B=8, lf=1, dtype="f32", seg=[0, 0, 1, 40, 40, 119, 120]),  # empty and 1-atom segments
    dict(N=72, L=4, C=16, H=2, B=8, lf=2, dtype="f32"),        # degree-2 filter
    dict(N=64, L=4, C=128, H=8, B=8, lf=1, dtype="bf16"),      # two waves per target
    dict(N=64, L=2, C=128, H=4, B=8, lf=2, dtype="f32"),
    dict(N=33, L=1, C=256, H=8, B=8, lf=1, dtype="bf16"),      # four waves per target
    dict(N=40, L=2, C=48, H=3, B=8, lf=1, dtype="f32"),        # idle lanes in the only wave
])
def test_shapes_and_filter_degrees(torch_cuda, kw):
    run_nonlinear(torch_cuda, _custom(5, **kw))


def test_large_molecules_at_the_benchmark_shape_sampled(torch_cuda):
    from paper_2601_16622_amd import workloads as W
    wl = W.by_name("large", 0)
    tg = np.random.default_rng(2).choice(wl["pos"].shape[0], 200, replace=False).astype(np.int32)
    run_nonlinear(torch_cuda, wl, tg)


def test_scaling_point_sampled(torch_cuda):
    from paper_2601_16622_amd import workloads as W
    wl = W.by_name("scaling", 0)
    tg = np.random.default_rng(4).choice(10_000, 100, replace=False).astype(np.int32)
    run_nonlinear(torch_cuda, wl, tg)


def test_periodic_boxes(torch_cuda):
    from paper_2601_16622_amd import workloads as W
    wl = W.periodic_boxes((500, 300), seed=6, L=2, C=64, H=4, B=8, cutoff=5.0, dtype="bf16")
    run_nonlinear(torch_cuda, wl)


def test_limits_and_empty_input(torch_cuda):
    from paper_2601_16622_amd import binding as B
    wl = _custom(5, N=33, L=1, C=128, H=1, B=8, lf=1, dtype="bf16")   # a head wider than a wave: not built
    P = B.Problem(wl)
    try:
        P.build_cells()
        with pytest.raises(B.E2fError) as e:
            P.forward_nonlinear()
        assert e.value.code == 2
    finally:
        P.close()
    wl = _custom(5, N=40, L=2, C=32, H=2, B=8, lf=1, dtype="f32")
    P = B.Problem(wl)
    try:
        P.build_cells()
        small = torch_cuda.empty(256, dtype=torch_cuda.uint8, device=P.device)
        with pytest.raises(B.E2fError) as e:
            B.e2f_attn_forward_nonlinear(P.ctx, P.cells, P.pos, P.h, P.seg, P.weights, P.out, small)
        assert e.value.code == 3
    finally:
        P.close()
