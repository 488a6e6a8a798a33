"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle, element by element on the same seeded
inputs.  Bar: neighbour sets identical; relative L2 error of the output <= 1e-4 for fp32 features and <= 2e-2 for
bf16 features with fp32 accumulation."""
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


def atom_errors(got, ref):
    """Relative L2 error of every atom's own output row (atoms with a zero reference: absolute error)."""
    d = np.linalg.norm((got - ref).reshape(ref.shape[0], -1), axis=1)
    r = np.linalg.norm(ref.reshape(ref.shape[0], -1), axis=1)
    return np.where(r > 0, d / np.where(r > 0, r, 1.0), d)


def run_case(torch, wl, targets=None, check_materialized=True, message_mode="dense", attention="auto", flags=0):
    import oracle as O
    from paper_2601_16622_amd import binding as B
    cfg = wl["cfg"]
    P = B.Problem(wl, attention=attention, flags=flags)
    try:
        P.build_cells()
        deg, offs, idx = P.neighbors()
        o_offs, o_idx = O.neighbor_list(wl["pos"], wl["seg"], np.float32(cfg["cutoff"]), use_cells=P.N > 3000)
        assert np.array_equal(offs, o_offs), "neighbour counts differ"
        assert np.array_equal(idx, o_idx), "neighbour sets differ"
        ref = O.attn_forward(cfg, wl["pos"], wl["h"], wl["seg"], wl["weights"], targets=targets, nbr=(o_offs, o_idx),
                             message_mode=message_mode)
        sel = slice(None) if targets is None else targets
        P.out.fill_(float("nan"))
        P.forward()
        torch.cuda.synchronize()
        fused = P.out.cpu().numpy().astype(np.float64)
        assert np.isfinite(fused).all()
        err = rel_l2(fused[sel], ref)
        assert err <= TOL[cfg["dtype"]], f"fused rel L2 {err}"
        # no single atom may hide in the norm over all of them (a wrong partial tile, a surface cell)
        worst = atom_errors(fused[sel], ref)
        assert worst.max() <= 5 * TOL[cfg["dtype"]], f"atom {int(np.argmax(worst))}: rel L2 {worst.max()}"
        for l in range(cfg["L"] + 1):   # no degree may hide behind the others
            if np.linalg.norm(ref[:, l * l:(l + 1) ** 2]) > 0:
                assert rel_l2(fused[sel][:, l * l:(l + 1) ** 2], ref[:, l * l:(l + 1) ** 2]) <= TOL[cfg["dtype"]]
        Ch = cfg["C"] // cfg["H"]
        if cfg["lf"] == 1 and Ch <= 64 and Ch & (Ch - 1) == 0:
            # the paper's factorized pipeline (node-level source/target products around Algorithm 1) gives the same result
            out_f = torch.full_like(P.out, float("nan"))
            P.forward_factorized(out_f)
            torch.cuda.synchronize()
            fact = out_f.cpu().numpy().astype(np.float64)
            assert np.isfinite(fact).all()
            errf = rel_l2(fact[sel], ref)
            assert errf <= TOL[cfg["dtype"]], f"factorized rel L2 {errf}"
        if check_materialized:
            out_m = torch.full_like(P.out, float("nan"))
            E, peak = P.forward_materialized(out_m)
            torch.cuda.synchronize()
            assert E == int(o_offs[-1]) and peak > 0
            errm = rel_l2(out_m.cpu().numpy().astype(np.float64)[sel], ref)
            assert errm <= 1e-4, f"materialized rel L2 {errm}"
        return err
    finally:
        P.close()


@pytest.mark.parametrize("name,seed", [("tiny", 0), ("tiny", 1), ("small", 0), ("large", 0)])
def test_named_configs_match_the_oracle(torch_cuda, name, seed):
    from paper_2601_16622_amd import workloads as W
    wl = W.by_name(name, seed)
    targets = None
    if name == "large":   # the dense fp64 route over all 4k atoms at L=4 takes minutes: sample targets
        targets = np.random.default_rng(1).choice(wl["pos"].shape[0], 400, replace=False).astype(np.int32)
    run_case(torch_cuda, wl, targets, message_mode="dense")


def test_scaling_point_every_target(torch_cuda):
    """The 10 000-atom box the benchmark times, same launch configuration: every target atom when the host has the
    threads for it (the oracle takes a few seconds on 8 or more), else 1 000 sampled ones."""
    import oracle as O
    from paper_2601_16622_amd import workloads as W
    wl = W.scaling_point(0)
    tg = None
    if O.num_threads() < 8:
        tg = np.random.default_rng(2).choice(10_000, 1000, replace=False).astype(np.int32)
    run_case(torch_cuda, wl, tg, message_mode="eaas")


def test_fp32_tile_kernel(torch_cuda):
    """fp32 features with heads of 16 channels run on the fp32 tile kernel (binary32 matrix instruction, the paper's own
    precision): the scaling point's box and shape in fp32 on 600 sampled targets, tolerance 1e-4 (128 MB of features:
    the projection runs on the weight-stationary fp32 kernel, the smaller cases below on the per-tile one); the same
    call on the vector-ALU kernel agrees; a box whose last tile is partial, with 13 radial functions; a dense
    core whose tiles do not fit the candidate list and go to the vector-ALU kernel, inside a sparse shell that does."""
    import oracle as O
    from paper_2601_16622_amd import binding as B, workloads as W
    wl = W.box(10_000, 0, dtype="f32")
    tg = large_n_targets(wl["pos"], 6.0, 400, 5)
    run_case(torch_cuda, wl, tg, check_materialized=False, message_mode="eaas")
    outs = []
    for att in ("tile", "valu"):
        P = B.Problem(wl, attention=att)
        P.build_cells()
        outs.append(P.forward().clone())
        P.close()
    torch_cuda.cuda.synchronize()
    d = (outs[0] - outs[1]).double().norm() / outs[1].double().norm()
    assert 0 < float(d) <= 1e-5, float(d)   # different kernels, same numbers to rounding
    run_case(torch_cuda, _custom(7, 333 + 6, 3, 64, 4, 13, 1, "f32", cutoff=3.5, side=9.0, seg=[0, 7, 8, 150, 339]),
             message_mode="eaas")
    rng = np.random.default_rng(14)
    cfg = dict(L=1, C=32, H=2, B=8, lf=1, cutoff=4.0, dtype="f32")
    mixed = np.concatenate([W.dart_throw_box(rng, 1500, 6.0, min_sep=0.3, origin=(5.0, 5.0, 5.0)),
                            W.dart_throw_box(rng, 250, 16.0, min_sep=1.5)])
    run_case(torch_cuda, W._pack(cfg, [mixed], rng, elements=False), check_materialized=False, message_mode="eaas")


def large_n_targets(pos, cutoff, n_random, seed):
    """Sampled targets of a big box: random atoms, the atoms of the box's last corner (the last cells of the sorted
    order, so the last tile of 16 slots is among them), and atoms next to the faces (surface cells, few neighbours)."""
    rng = np.random.default_rng(seed)
    N = pos.shape[0]
    hi, lo = pos.max(axis=0), pos.min(axis=0)
    corner = np.nonzero((pos[:, 2] > hi[2] - 1.001 * cutoff) & (pos[:, 1] > hi[1] - 1.001 * cutoff) &
                        (pos[:, 0] > hi[0] - 2.1 * cutoff))[0]
    face = np.nonzero(((pos - lo) < 0.5).any(axis=1) | ((hi - pos) < 0.5).any(axis=1))[0]
    face = rng.choice(face, min(150, face.size), replace=False)
    rnd = rng.choice(N, n_random, replace=False)
    return np.unique(np.concatenate([rnd, corner, face])).astype(np.int32)


@pytest.mark.parametrize("N", [20_000, 20_011, 50_000, 100_000])
def test_large_n_sampled(torch_cuda, N):
    """The Large-N regime (20k, 50k, 100k atoms at the same density) and a box whose last tile is partial: neighbour
    sets of every atom, the output on 500 random targets plus the last corner and the faces; fused path only."""
    from paper_2601_16622_amd import workloads as W
    wl = W.box(N, seed=3)
    tg = large_n_targets(wl["pos"], wl["cfg"]["cutoff"], 500, seed=N)
    assert tg.size >= 600
    run_case(torch_cuda, wl, tg, check_materialized=False, message_mode="eaas")


def _custom(seed, N, L, C, H, B, lf, dtype, cutoff=3.0, side=6.0, seg=None):
    from paper_2601_16622_amd import workloads as W
    rng = np.random.default_rng(seed)
    cfg = dict(L=L, C=C, H=H, B=B, lf=lf, cutoff=cutoff, dtype=dtype)
    pos = W.dart_throw_box(rng, N, side)
    wl = W._pack(cfg, [pos], rng, elements=False)
    if seg is not None:
        wl["seg"] = np.asarray(seg, dtype=np.int32)
    return wl


@pytest.mark.parametrize("kw", [
    dict(N=50, L=0, C=32, H=4, B=4, lf=0, dtype="f32"),        # scalar attention
    dict(N=77, L=2, C=64, H=4, B=1, lf=0, dtype="f32"),        # lf = 0 with higher degrees, a single radial function
    dict(N=61, L=3, C=32, H=2, B=8, lf=1, dtype="bf16"),       # odd L, bf16, ragged last MFMA tile
    dict(N=90, L=4, C=64, H=8, B=16, lf=1, dtype="f32"),       # L = 4 in fp32, one channel per lane
    dict(N=33, L=1, C=256, H=8, B=8, lf=1, dtype="bf16"),      # four channels per lane
    dict(N=120, L=2, C=16, H=1, B=8, lf=1, dtype="f32", seg=[0, 0, 1, 40, 40, 119, 120]),  # empty and 1-atom segments
    dict(N=70, L=2, C=64, H=4, B=8, lf=1, dtype="bf16"),       # matrix-core path with the low tile only
    dict(N=45, L=1, C=32, H=2, B=3, lf=1, dtype="bf16"),       # matrix-core path, L = 1
    dict(N=150, L=4, C=16 * 1, H=1, B=8, lf=1, dtype="f32"),   # one head of 16 channels in fp32 (vector-ALU path)
    dict(N=83, L=4, C=64, H=4, B=8, lf=1, dtype="bf16", seg=[0, 30, 30, 83]),  # matrix-core path, 4 heads, segments
    dict(N=64, L=2, C=64, H=2, B=8, lf=1, dtype="bf16"),       # bf16 with 32-channel heads: vector-ALU path, bf16 v
    dict(N=64, L=3, C=64, H=4, B=8, lf=0, dtype="bf16"),       # bf16, lf = 0
    dict(N=60, L=2, C=32, H=2, B=8, lf=2, dtype="f32"),        # degree-2 filter, vector-ALU path
    dict(N=72, L=4, C=16, H=2, B=8, lf=2, dtype="f32"),        # degree-2 filter, L = 4
    dict(N=90, L=4, C=64, H=4, B=8, lf=2, dtype="bf16"),       # degree-2 filter on the matrix-core path
    dict(N=50, L=2, C=32, H=2, B=8, lf=2, dtype="bf16"),       # degree-2 filter, low tile only
    dict(N=200, L=4, C=64, H=4, B=16, lf=1, dtype="bf16"),     # tile kernels with 16 radial basis functions
    dict(N=150, L=2, C=32, H=2, B=11, lf=1, dtype="bf16"),     # ... and with 11
    dict(N=300, L=4, C=256, H=16, B=8, lf=1, dtype="bf16", side=8.5),    # 256 channels on the tile kernels (plain projection + relayout)
    dict(N=210, L=2, C=48, H=3, B=8, lf=1, dtype="f32", side=7.0),       # 48 channels in three heads: the fp32 tile kernel
])
def test_other_shapes_and_degenerate_inputs(torch_cuda, kw):
    run_case(torch_cuda, _custom(5, **kw))


@pytest.mark.parametrize("kernel", ["tile", "pair", "valu"])
@pytest.mark.parametrize("name", ["large", "scaling", "odd", "odd_b13"])
def test_each_attention_kernel_matches_the_oracle(torch_cuda, name, kernel):
    """The three forms of the attention stage on the same bf16 inputs, selected through the configuration: the tile form
    (16 targets x 32 candidates on the matrix cores, linear factorization of the degree-1 filter; the default where it
    applies), the per-pair matrix-core form and the ALU form; multi-segment tiles, partial last tile, L_max < 4."""
    from paper_2601_16622_amd import workloads as W
    if name == "large":
        wl = W.by_name("large", 0)
        tg = np.random.default_rng(1).choice(wl["pos"].shape[0], 300, replace=False).astype(np.int32)
    elif name == "scaling":
        wl = W.scaling_point(0)
        tg = np.random.default_rng(2).choice(10_000, 200, replace=False).astype(np.int32)
    else:
        wl = _custom(5, 333, 2, 64, 4, 13 if name == "odd_b13" else 5, 1, "bf16", cutoff=3.5, side=9.0, seg=[0, 7, 8, 150, 333])
        tg = None
    run_case(torch_cuda, wl, tg, check_materialized=False, message_mode="eaas", attention=kernel)


def _capped_case(torch, wl, K, attention="auto"):
    """(Problem, oracle neighbour lists capped to the K nearest, oracle output for them)."""
    import oracle as O
    from paper_2601_16622_amd import binding as B
    cfg = wl["cfg"]
    P = B.Problem(wl, attention=attention)
    P.build_cells()
    offs, idx = O.neighbor_list(wl["pos"], wl["seg"], np.float32(cfg["cutoff"]), use_cells=False)
    c_offs, c_idx = O.cap_neighbors(wl["pos"], offs, idx, K)
    ref = O.attn_forward(cfg, wl["pos"], wl["h"], wl["seg"], wl["weights"], nbr=(c_offs, c_idx), message_mode="eaas")
    return P, (offs, idx), (c_offs, c_idx), ref


@pytest.mark.parametrize("K", [5, 16])
def test_neighbor_table_holds_the_k_nearest(torch_cuda, K):
    """e2f_build_neighbor_table against the oracle's selection rule: same set in every row (order within a row is free),
    same counts, -1 padding; segments, a ragged last row and atoms with fewer than K neighbours included."""
    wl = _custom(11, 700, 1, 32, 2, 4, 1, "f32", cutoff=3.2, side=13.0, seg=[0, 3, 4, 350, 700])
    P, (offs, idx), (c_offs, c_idx), _ = _capped_case(torch_cuda, wl, K)
    try:
        table, count = P.neighbor_table(K)
        torch_cuda.cuda.synchronize()
        table, count = table.cpu().numpy(), count.cpu().numpy()
        deg = np.diff(offs)
        assert np.array_equal(count, np.minimum(deg, K))
        assert (deg > K).any() and (deg < K).any()
        for i in range(P.N):
            row = table[i]
            assert np.array_equal(np.sort(row[:count[i]]), c_idx[c_offs[i]:c_offs[i + 1]]), i
            assert (row[count[i]:] == -1).all()
    finally:
        P.close()


def test_neighbor_table_with_more_neighbours_than_the_selection_keeps_on_chip(torch_cuda):
    """700 atoms inside one cutoff sphere: every atom has 699 neighbours, above the 512 keys the selection kernel keeps
    in LDS, so the per-digit stencil walk is used."""
    from paper_2601_16622_amd import workloads as W
    rng = np.random.default_rng(21)
    cfg = dict(L=1, C=32, H=2, B=4, lf=1, cutoff=9.0, dtype="f32")
    wl = W._pack(cfg, [rng.uniform(0.0, 5.0, size=(700, 3)).astype(np.float32)], rng, elements=False)
    K = 40
    P, (offs, idx), (c_offs, c_idx), _ = _capped_case(torch_cuda, wl, K)
    try:
        assert np.diff(offs).min() > 512
        table, count = P.neighbor_table(K)
        torch_cuda.cuda.synchronize()
        table, count = table.cpu().numpy(), count.cpu().numpy()
        assert (count == K).all()
        for i in range(P.N):
            assert np.array_equal(np.sort(table[i]), c_idx[c_offs[i]:c_offs[i + 1]]), i
    finally:
        P.close()


@pytest.mark.parametrize("kernel", ["tile", "pair", "valu"])
def test_capped_forward_matches_the_oracle(torch_cuda, kernel):
    """max_neighbors = 12 (about a third of the mean degree) through each attention kernel."""
    wl = _custom(12, 500, 3, 64, 4, 6, 1, "bf16", cutoff=4.0, side=11.0, seg=[0, 200, 500])
    P, _, _, ref = _capped_case(torch_cuda, wl, 12, attention=kernel)
    try:
        P.out.fill_(float("nan"))
        P.forward_capped(12)
        torch_cuda.cuda.synchronize()
        got = P.out.cpu().numpy().astype(np.float64)
        assert rel_l2(got, ref) <= TOL["bf16"]
        P.forward()   # and the cap really changes the result
        torch_cuda.cuda.synchronize()
        assert rel_l2(P.out.cpu().numpy().astype(np.float64), ref) > 0.05
    finally:
        P.close()


def test_fcc_lattice_with_equidistant_neighbours(torch_cuda):
    """Sites of an FCC lattice (the paper's scaling systems): shells of exactly equidistant neighbours, pair vectors
    along the axes and face diagonals (poles of the aligning rotation); full neighbourhoods and a cap that cuts
    through a shell, where only the index tie rule decides."""
    from paper_2601_16622_amd import workloads as W
    wl = W.fcc_subsample(600, 0, L=2, C=64, H=4, dtype="bf16")
    run_case(torch_cuda, wl, check_materialized=True, message_mode="eaas")
    P, (offs, _), _, ref = _capped_case(torch_cuda, wl, 20)   # the third shell (24 sites) is cut
    try:
        assert np.diff(offs).max() > 40
        P.forward_capped(20)
        torch_cuda.cuda.synchronize()
        assert rel_l2(P.out.cpu().numpy().astype(np.float64), ref) <= TOL["bf16"]
    finally:
        P.close()


def test_capped_forward_fp32_and_no_effect_above_the_degree(torch_cuda):
    wl = _custom(13, 300, 2, 32, 2, 8, 1, "f32", cutoff=3.5, side=9.0)
    P, (offs, _), _, ref = _capped_case(torch_cuda, wl, 7)
    try:
        P.forward_capped(7)
        torch_cuda.cuda.synchronize()
        assert rel_l2(P.out.cpu().numpy().astype(np.float64), ref) <= TOL["f32"]
        full = P.forward().clone()
        P.forward_capped(int(np.diff(offs).max()))   # a cap at the largest degree changes nothing
        torch_cuda.cuda.synchronize()
        # (the uncapped call runs on the fp32 tile kernel here, the capped one on the vector-ALU kernel: the same
        # numbers to rounding; on one kernel, as in the bf16 test of the cap, they are the same bits)
        assert float((full - P.out).double().norm() / full.double().norm()) <= 1e-5
        Pv = __import__("paper_2601_16622_amd.binding", fromlist=["Problem"]).Problem(wl, attention="valu")
        try:
            Pv.build_cells()
            full_v = Pv.forward().clone()
            Pv.forward_capped(int(np.diff(offs).max()))
            torch_cuda.cuda.synchronize()
            assert torch_cuda.equal(full_v, Pv.out)
        finally:
            Pv.close()
    finally:
        P.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_forward_over_a_padded_table(torch_cuda, dtype):
    """e2f_attn_forward_table: the library's own table, and a hand-made one (a random subset of the true neighbours in
    shuffled order, with holes, a self entry, an atom beyond the cutoff and repeated padding) against the oracle run on
    the same lists; fp32 features go through the vector-ALU kernel, bf16 ones through the tile kernel (the table as a
    mask on the tiles' candidate lists)."""
    import oracle as O
    wl = _custom(14, 260, 2, 32, 2, 8, 1, dtype, cutoff=3.5, side=8.5, seg=[0, 100, 260])
    K = 16
    P, (offs, idx), (c_offs, c_idx), ref = _capped_case(torch_cuda, wl, K)
    try:
        table, _ = P.neighbor_table(K)
        out = torch_cuda.full_like(P.out, float("nan"))
        P.forward_table(table, out)
        torch_cuda.cuda.synchronize()
        assert rel_l2(out.cpu().numpy().astype(np.float64), ref) <= TOL[dtype]
        rng = np.random.default_rng(5)
        hand = -np.ones((P.N, K + 3), dtype=np.int32)
        rows, h_off = [], np.zeros(P.N + 1, dtype=np.int64)
        for i in range(P.N):
            nb = idx[offs[i]:offs[i + 1]]
            pick = rng.permutation(nb)[:rng.integers(0, min(len(nb), K) + 1)]
            slots = rng.permutation(K + 3)[:len(pick)]
            hand[i, slots] = pick
            free = np.setdiff1d(np.arange(K + 3), slots)
            hand[i, free[0]] = i            # a self entry is ignored
            s0, s1 = wl["seg"][np.searchsorted(wl["seg"], i, side="right") - 1], wl["seg"][np.searchsorted(wl["seg"], i, side="right")]
            far = [j for j in range(s0, s1) if j != i and j not in nb]
            if far:
                hand[i, free[1]] = far[rng.integers(len(far))]   # and so is an atom outside the cutoff
            rows.append(np.sort(pick).astype(np.int32))
            h_off[i + 1] = h_off[i] + len(pick)
        h_idx = np.concatenate(rows).astype(np.int32)
        cfg = wl["cfg"]
        ref2 = O.attn_forward(cfg, wl["pos"], wl["h"], wl["seg"], wl["weights"], nbr=(h_off, h_idx), message_mode="eaas")
        P.forward_table(torch_cuda.from_numpy(hand).to(P.device), out)
        torch_cuda.cuda.synchronize()
        assert rel_l2(out.cpu().numpy().astype(np.float64), ref2) <= TOL[dtype]
    finally:
        P.close()


def test_isolated_atoms_and_crowded_cells(torch_cuda):
    """Atoms with no neighbour give zeros; a target with more neighbours than one LDS list holds still matches."""
    from paper_2601_16622_amd import workloads as W
    rng = np.random.default_rng(9)
    cfg = dict(L=1, C=16, H=2, B=8, lf=1, cutoff=4.0, dtype="f32")
    crowd = W.dart_throw_box(rng, 420, 6.0, min_sep=0.5)            # ~250 neighbours for central atoms
    far = np.array([[100.0, 0, 0], [0, 200.0, 0], [-300.0, -300.0, 50.0]], dtype=np.float32)
    wl = W._pack(cfg, [np.concatenate([crowd, far])], rng, elements=False)
    import oracle as O
    offs, _ = O.neighbor_list(wl["pos"], wl["seg"], np.float32(4.0))
    assert np.diff(offs).max() > 192 and np.all(np.diff(offs)[-3:] == 0)
    run_case(torch_cuda, wl)
    from paper_2601_16622_amd import binding as B
    P = B.Problem(wl)
    P.build_cells()
    P.forward()
    torch_cuda.cuda.synchronize()
    assert torch_cuda.all(P.out[-3:] == 0)
    P.close()


def test_tile_kernel_with_lists_longer_than_the_shared_list_area(torch_cuda):
    """1500 atoms in a 6 A box (bf16, heads of 16: the tile kernel): central atoms have over 1000 neighbours, so their
    tiles keep more slot groups than a tile's shared candidate list holds (192 entries) and more than one batch of
    the list in LDS (256): those tiles build their lists per head, in several batches; a sparse cluster beside them
    uses the shared lists."""
    from paper_2601_16622_amd import workloads as W
    rng = np.random.default_rng(10)
    cfg = dict(L=1, C=32, H=2, B=8, lf=1, cutoff=4.0, dtype="bf16")
    crowd = W.dart_throw_box(rng, 1500, 6.0, min_sep=0.3)
    sparse = W.dart_throw_box(rng, 200, 14.0, origin=(40.0, 0.0, 0.0))
    wl = W._pack(cfg, [crowd, sparse], rng, elements=False)
    import oracle as O
    offs, _ = O.neighbor_list(wl["pos"], wl["seg"], np.float32(4.0))
    assert np.diff(offs)[:1500].max() > 4 * 256 and np.diff(offs)[1500:].max() < 100
    run_case(torch_cuda, wl, check_materialized=False)


def test_result_is_deterministic_and_order_equivariant(torch_cuda):
    from paper_2601_16622_amd import binding as B, workloads as W
    wl = W.small_molecules(2, n_mol=6)
    P = B.Problem(wl)
    P.build_cells()
    a = P.forward().clone()
    P.build_cells()
    b = P.forward().clone()
    assert torch_cuda.equal(a, b)
    # permuting atoms inside a segment permutes the rows of the output (values may differ by rounding order only)
    s0, s1 = int(wl["seg"][1]), int(wl["seg"][2])
    perm = np.arange(wl["pos"].shape[0])
    perm[s0:s1] = perm[s0:s1][::-1]
    wl2 = dict(wl, pos=wl["pos"][perm], h=wl["h"][perm])
    P2 = B.Problem(wl2)
    P2.build_cells()
    c = P2.forward()
    torch_cuda.cuda.synchronize()
    ref = a.cpu().numpy()[perm]
    assert rel_l2(c.cpu().numpy(), ref) < 1e-5
    P.close()
    P2.close()


@pytest.mark.parametrize("name", ["large", "scaling", "pbox2500"])
def test_shared_candidate_lists_and_lists_built_per_head_agree(torch_cuda, name):
    """The tile kernel reads candidate lists built once per tile (all heads) or builds them per (tile, head): the same
    pairs either way.  The order of the candidates differs, and with it the softmax reference that the bf16 weights
    are rounded against, so the two agree to bf16 rounding noise (well inside the tolerance against the oracle)."""
    from paper_2601_16622_amd import binding as B
    from paper_2601_16622_amd import workloads as W
    wl = W.by_name(name, 0)
    P = B.Problem(wl)
    Q = B.Problem(wl, flags=B.E2F_FLAG_TILE_LISTS_PER_HEAD)
    try:
        P.build_cells()
        P.forward()
        Q.build_cells()
        Q.out.fill_(float("nan"))
        Q.forward()
        torch_cuda.cuda.synchronize()
        shared, per_head = P.out.clone(), Q.out.clone()
        assert torch_cuda.isfinite(shared).all() and torch_cuda.isfinite(per_head).all()
        assert float((shared - per_head).norm() / per_head.norm()) < 5e-3
        # a neighbour cap prunes the lists with every target's own reach
        a = P.forward_capped(24, torch_cuda.empty_like(P.out))
        b = Q.forward_capped(24, torch_cuda.empty_like(Q.out))
        torch_cuda.cuda.synchronize()
        assert float((a - b).norm() / b.norm()) < 5e-3
    finally:
        P.close()
        Q.close()


@pytest.mark.parametrize("name", ["tiny", "odd_bf16"])
def test_step_replays_from_a_captured_graph(torch_cuda, name):
    """e2f_build_cells + e2f_attn_forward allocate nothing, never synchronise and clear their counters with kernels, so a
    step can be captured into a graph; every replay (with eager work and synchronisations in between, and with the
    positions changed before the last one) gives the bits of the eager call."""
    from paper_2601_16622_amd import binding as B, workloads as W
    torch = torch_cuda
    wl = W.tiny(3) if name == "tiny" else _custom(31, 333, 2, 64, 4, 5, 1, "bf16", cutoff=3.5, side=9.0, seg=[0, 150, 333])
    P = B.Problem(wl)
    try:
        def step():
            P.build_cells()
            P.forward()
        step()
        torch.cuda.synchronize()
        eager = P.out.clone()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            step()   # warm-up on the capture stream
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.synchronize()
        for rep in range(3):
            P.out.fill_(float("nan"))
            _ = (P.h.float() * 2).sum().item()   # eager work and a synchronisation between replays
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(P.out, eager), rep
        # new positions in the same buffers: the replay follows them (cells are rebuilt inside the graph)
        P.pos.add_(torch.randn_like(P.pos) * 0.05)
        graph.replay()
        torch.cuda.synchronize()
        replayed = P.out.clone()
        step()
        torch.cuda.synchronize()
        assert torch.equal(P.out, replayed)
    finally:
        P.close()


def test_fused_activation_memory_is_linear_and_below_the_baseline(torch_cuda):
    from paper_2601_16622_amd import binding as B, workloads as W
    wl = W.box(3000, seed=4)
    P = B.Problem(wl)
    P.build_cells()
    torch_cuda.cuda.synchronize()
    torch_cuda.cuda.reset_peak_memory_stats()
    before = torch_cuda.cuda.memory_allocated()
    P.forward()
    torch_cuda.cuda.synchronize()
    assert torch_cuda.cuda.max_memory_allocated() == before       # the fused call allocates nothing
    E, peak = P.forward_materialized(torch_cuda.empty_like(P.out))
    assert peak > 5 * P.activation_bytes()
    P.close()
