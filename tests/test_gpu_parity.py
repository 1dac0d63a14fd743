"""GPU parity tests: the HIP path, called through the C ABI, against the CPU oracle on the
same seeded inputs.  Integer results (tables, neighbour / child lists, pooling switches,
gathered columns) must match bit for bit; floating-point results must satisfy
    |gpu - oracle| <= tol * (|oracle| + rms(oracle)),  tol = 1e-4 for fp32.
"""
import numpy as np
import pytest

import synth_shapes as S

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
hch = pytest.importorskip("paper_1803_11385_amd")

TOL_F32 = 1e-4


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda")


def assert_close(got, want, tol=TOL_F32, what=""):
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    assert np.isfinite(got).all(), what
    rms = float(np.sqrt((want ** 2).mean())) if want.size else 0.0
    err = np.abs(got - want)
    bound = tol * (np.abs(want) + rms)
    worst = float((err / np.maximum(bound, 1e-300)).max()) if want.size else 0.0
    assert worst <= 1.0, f"{what}: max err/bound = {worst:.3g}, max abs err = {err.max():.3g}, rms = {rms:.3g}"


def workspace(nbytes):
    # every byte 0xFF (NaN as a float, -1 as an index): a read of something the library did not write shows
    t = torch.full((max(nbytes, 256) + 256,), 255, dtype=torch.uint8, device="cuda")
    off = (-t.data_ptr()) % 256
    return t[off: off + max(nbytes, 256)]


class Case:
    """Geometry + both implementations' levels."""

    def __init__(self, oracle, coords, offs, u, n_levels):
        self.coords, self.offs, self.u = coords, np.asarray(offs, np.int64), u
        self.olv = oracle.build_hierarchy(coords, offs, u, n_levels)
        self.glv = hch.hch_build_levels(coords, offs, u, n_levels)
        torch.cuda.synchronize()


@pytest.fixture(scope="module")
def case_sphere(oracle):
    coords, normals = S.sphere_shell_32()
    c = Case(oracle, coords, [0, coords.shape[0]], 32, 2)
    c.normals = normals
    return c


@pytest.fixture(scope="module")
def case_batch64(oracle):
    coords, offs, normals = S.config_batch(2, with_normals=True)
    c = Case(oracle, coords, offs, 64, 3)
    c.normals = normals
    return c


@pytest.fixture(scope="module")
def case_small(oracle):
    # several GEMM tiles and a ragged tail, small enough for the oracle's column matrix
    coords, offs, _ = S.config_batch(3, batch=4, u=64)
    return Case(oracle, coords, offs, 64, 3)


# --------------------------------------------------------------------------------------
# tables and index lists: bit-exact
# --------------------------------------------------------------------------------------

@pytest.mark.parametrize("name", ["case_sphere", "case_batch64", "case_small"])
def test_tables_and_index_lists_bit_exact(request, oracle, name):
    case = request.getfixturevalue(name)
    for l, L in enumerate(case.olv):
        info = case.glv.info(l)
        assert np.array_equal(info.mbar, L.mbar) and np.array_equal(info.rbar, L.rbar)
        assert np.array_equal(info.M, L.M) and np.array_equal(info.R, L.R) and np.array_equal(info.N, L.N)
        assert np.array_equal(info.device_H(), L.H)
        assert np.array_equal(info.device_T(), L.T)
        assert np.array_equal(info.device_Phi(), L.Phi)
        assert np.array_equal(info.device_V(), L.V)
        assert np.array_equal(info.device_coords(), L.coords)
        assert np.array_equal(info.device_nbr27(), oracle.neighbours(L)), f"nbr27 level {l}"
        if l > 0:
            assert np.array_equal(info.device_child8(), oracle.children(case.olv[l - 1], L)), f"child8 level {l}"


@pytest.mark.parametrize("name", ["case_sphere", "case_batch64", "case_small"])
def test_pattern_order_and_tile_taps(request, oracle, name):
    """The order in which the fused products walk a level and the taps each of its 64-row tiles
    has: a permutation of the level's voxels, sorted stably by a 6-bit key (one bit per pair of
    opposite edge-adjacent neighbours, taps k and 26-k for k = 1, 3, .., 11: set if either
    exists), and per tile exactly the union of its voxels' neighbour sets, all derived from the
    oracle's neighbour lists."""
    case = request.getfixturevalue(name)
    for l, L in enumerate(case.olv):
        info = case.glv.info(l)
        valid = oracle.neighbours(L) >= 0
        key = np.zeros(L.Ntot, np.int64)
        for k in range(1, 13, 2):
            key = key * 2 + (valid[:, k] | valid[:, 26 - k])
        order = info.device_row_order()
        assert np.array_equal(order, np.argsort(key, kind="stable")), f"level {l}"
        mask = valid.astype(np.int64) @ (1 << np.arange(27, dtype=np.int64))
        pad = np.zeros(-(-L.Ntot // 64) * 64, np.int64)
        pad[:L.Ntot] = mask[order]
        assert np.array_equal(info.device_tile_taps().astype(np.int64), np.bitwise_or.reduce(pad.reshape(-1, 64), axis=1)), f"level {l}"


def test_neighbour_rebuild_is_idempotent(oracle, case_batch64):
    case = case_batch64
    for l in range(3):
        hch.hch_build_neighbours(case.glv, l)
    hch.hch_build_neighbours_range(case.glv, 1, 2)
    hch.hch_build_neighbours_range(case.glv, 0, 0)
    with pytest.raises(hch.HchError):
        hch.hch_build_neighbours_range(case.glv, 2, 2)
    torch.cuda.synchronize()
    assert np.array_equal(case.glv.info(1).device_nbr27(), oracle.neighbours(case.olv[1]))
    assert np.array_equal(case.glv.info(2).device_child8(), oracle.children(case.olv[1], case.olv[2]))


# --------------------------------------------------------------------------------------
# hash2col / col2hash
# --------------------------------------------------------------------------------------

def _oracle_col(oracle, L, X):
    """oracle's (c*27) x N column matrix rearranged to the library's [N][27*c] (k-major)."""
    c = X.shape[1]
    Dt = oracle.hash2col(L, L, oracle.to_paper_X(X))
    return np.ascontiguousarray(Dt.reshape(c, 27, L.Ntot).transpose(2, 1, 0).reshape(L.Ntot, 27 * c))


@pytest.mark.parametrize("c_in", [3, 4, 32])
def test_hash2col_bit_exact(oracle, case_batch64, c_in):
    case = case_batch64
    L = case.olv[1]
    X = S.gaussian((L.Ntot, c_in), 1.0, 11)
    col = torch.full((L.Ntot, 27 * c_in), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_hash2col(case.glv, 1, hch.HCH_F32, dev(X), c_in, 0, L.Ntot, col)
    want = _oracle_col(oracle, L, X).astype(np.float32)
    assert np.array_equal(col.cpu().numpy(), want)
    # a row range in the middle
    r0, rows = 1000, 777
    part = torch.full((rows, 27 * c_in), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_hash2col(case.glv, 1, hch.HCH_F32, dev(X), c_in, r0, rows, part)
    assert np.array_equal(part.cpu().numpy(), want[r0:r0 + rows])


def test_hash2col_bf16_bit_exact(oracle, case_batch64):
    case = case_batch64
    L = case.olv[1]
    for c_in in (8, 5):
        X = S.to_bf16_grid(S.gaussian((L.Ntot, c_in), 1.0, 12))
        bits = S.bf16_bits(X)
        col = torch.full((L.Ntot, 27 * c_in), 0x7FC0, dtype=torch.int16, device="cuda")
        hch.hch_hash2col(case.glv, 1, hch.HCH_BF16, dev(bits.view(np.int16)), c_in, 0, L.Ntot, col)
        want = S.bf16_bits(_oracle_col(oracle, L, X).astype(np.float32))
        assert np.array_equal(col.cpu().numpy().view(np.uint16), want)


@pytest.mark.parametrize("c_in", [3, 8])
def test_col2hash(oracle, case_small, c_in):
    case = case_small
    L = case.olv[0]
    dcol = S.gaussian((L.Ntot, 27 * c_in), 1.0, 13)
    dX = torch.full((L.Ntot, c_in), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_col2hash(case.glv, 0, dev(dcol), c_in, dX)
    dDt = dcol.astype(np.float64).reshape(L.Ntot, 27, c_in).transpose(2, 1, 0).reshape(c_in * 27, L.Ntot)
    want = oracle.col2hash(L, L, dDt, c_in).T
    assert_close(dX.cpu().numpy(), want, what="col2hash")
    # run-to-run reproducibility
    dX2 = torch.empty_like(dX)
    hch.hch_col2hash(case.glv, 0, dev(dcol), c_in, dX2)
    assert torch.equal(dX, dX2)


# --------------------------------------------------------------------------------------
# convolution forward and backward
# --------------------------------------------------------------------------------------

ALGOS = [hch.HCH_ALGO_COLUMNS, hch.HCH_ALGO_FUSED, hch.HCH_ALGO_FUSED_DENSE]
ALGO_IDS = ["columns", "fused", "fused-dense"]


def _conv_fwd_gpu(case, level, X, W, ws_bytes=None, algo=hch.HCH_ALGO_COLUMNS):
    n, c_in = X.shape
    c_out = W.shape[2]
    if ws_bytes is None:
        ws_bytes = hch.hch_conv_workspace_bytes(case.glv, level, c_in, c_out, hch.HCH_F32, hch.HCH_WS_FWD, algo)
    ws = workspace(ws_bytes)
    Y = torch.full((n, c_out), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_conv_fwd(case.glv, level, hch.HCH_F32, dev(X), dev(W), Y, c_in, c_out, ws, algo)
    return Y.cpu().numpy()


@pytest.mark.parametrize("algo", ALGOS, ids=ALGO_IDS)
def test_conv_fwd_sphere_3_to_16(oracle, case_sphere, algo):
    """Single shape, 32^3, 3 -> 16 channels, weights N(0, 0.1) seed 0, then max-pool to 16^3."""
    case = case_sphere
    L = case.olv[0]
    W = S.gaussian((27, 3, 16), 0.1, 0)
    Y = _conv_fwd_gpu(case, 0, case.normals, W, algo=algo)
    want = oracle.conv_fwd(L, oracle.to_paper_X(case.normals), oracle.to_paper_W(W))
    assert_close(Y, want.T, what="conv fwd sphere")
    # pool the GPU's own conv output on both sides: same fp32 inputs, so the switches must agree
    Yp = torch.empty((case.olv[1].Ntot, 16), dtype=torch.float32, device="cuda")
    sw = torch.empty((case.olv[1].Ntot, 16), dtype=torch.int32, device="cuda")
    hch.hch_pool_fwd(case.glv, 0, dev(Y), Yp, sw, 16)
    Po, swo = oracle.pool_max_fwd(L, case.olv[1], oracle.to_paper_X(Y))
    assert np.array_equal(sw.cpu().numpy(), swo.T)
    assert np.array_equal(Yp.cpu().numpy(), Po.T.astype(np.float32))


@pytest.mark.parametrize("algo", ALGOS, ids=ALGO_IDS)
def test_conv_fwd_batch64_4_to_32(oracle, case_batch64, algo):
    case = case_batch64
    L = case.olv[0]
    X = S.normals_plus_one(case.normals)
    W = S.gaussian((27, 4, 32), 0.05, 2000)
    want = oracle.conv_fwd(L, oracle.to_paper_X(X), oracle.to_paper_W(W)).T
    assert_close(_conv_fwd_gpu(case, 0, X, W, algo=algo), want, what="conv fwd 4->32")
    if algo != hch.HCH_ALGO_COLUMNS:
        return
    # the same through a workspace that forces several chunks
    small = hch.hch_conv_workspace_bytes(case.glv, 0, 4, 32, hch.HCH_F32, hch.HCH_WS_MIN)
    assert_close(_conv_fwd_gpu(case, 0, X, W, ws_bytes=small * 5 + 4096), want, what="conv fwd chunked")


@pytest.mark.parametrize("algo", ALGOS, ids=ALGO_IDS)
@pytest.mark.parametrize("c_in,c_out,level", [(32, 64, 0), (16, 32, 1), (5, 7, 1), (64, 128, 2), (8, 80, 2),
                                              (128, 256, 2), (4, 16, 0), (4, 32, 0), (4, 64, 1), (16, 4, 1),
                                              (32, 16, 1)])
def test_conv_fwd_and_gradients(oracle, case_small, c_in, c_out, level, algo):
    case = case_small
    L = case.olv[level]
    n = L.Ntot
    X = S.gaussian((n, c_in), 1.0, 21)
    W = S.he_weights(c_in, c_out, 22)
    G = S.gaussian((n, c_out), 1.0, 23)
    Xp, Wp, Gp = oracle.to_paper_X(X), oracle.to_paper_W(W), oracle.to_paper_X(G)

    assert_close(_conv_fwd_gpu(case, level, X, W, algo=algo), oracle.conv_fwd(L, Xp, Wp).T, what="fwd")

    ws = workspace(hch.hch_conv_workspace_bytes(case.glv, level, c_in, c_out, hch.HCH_F32, hch.HCH_WS_BWD_DATA, algo))
    dX = torch.full((n, c_in), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_conv_bwd_data(case.glv, level, hch.HCH_F32, dev(G), dev(W), dX, c_in, c_out, ws, algo)
    assert_close(dX.cpu().numpy(), oracle.conv_bwd_data(L, Gp, Wp, c_in).T, what="bwd data")

    ws = workspace(hch.hch_conv_workspace_bytes(case.glv, level, c_in, c_out, hch.HCH_F32, hch.HCH_WS_BWD_WEIGHT, algo))
    dW = torch.full((27, c_in, c_out), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_conv_bwd_weight(case.glv, level, hch.HCH_F32, dev(X), dev(G), dW, c_in, c_out, ws, algo)
    want_dW = oracle.from_paper_W(oracle.conv_bwd_weight(L, Xp, Gp), c_in)
    assert_close(dW.cpu().numpy(), want_dW, what="bwd weight")
    dW2 = torch.empty_like(dW)
    hch.hch_conv_bwd_weight(case.glv, level, hch.HCH_F32, dev(X), dev(G), dW2, c_in, c_out, ws, algo)
    assert torch.equal(dW, dW2)


# --------------------------------------------------------------------------------------
# caller order is the contract: the finest level's data index is the order of the caller's
# coordinates, whatever it is
# --------------------------------------------------------------------------------------

@pytest.fixture(scope="module")
def case_permuted(oracle):
    """The 64^3 / batch 32 workload with the voxels of every model in a seeded random order (the
    generator hands them out sorted by linear position)."""
    coords, offs, normals = S.config_batch(2, with_normals=True)
    rng = np.random.default_rng(2718)
    perm = np.concatenate([offs[v] + rng.permutation(int(offs[v + 1] - offs[v])) for v in range(len(offs) - 1)])
    c = Case(oracle, np.ascontiguousarray(coords[perm]), offs, 64, 3)
    c.normals = np.ascontiguousarray(normals[perm])
    c.perm = perm
    return c


def test_permuted_input_tables_and_lists(oracle, case_permuted, case_batch64):
    case = case_permuted
    for l, L in enumerate(case.olv):
        info = case.glv.info(l)
        assert np.array_equal(info.mbar, L.mbar) and np.array_equal(info.rbar, L.rbar)
        assert np.array_equal(info.M, L.M) and np.array_equal(info.R, L.R) and np.array_equal(info.N, L.N)
        assert np.array_equal(info.device_H(), L.H) and np.array_equal(info.device_T(), L.T)
        assert np.array_equal(info.device_Phi(), L.Phi) and np.array_equal(info.device_V(), L.V)
        assert np.array_equal(info.device_coords(), L.coords)
        nb = info.device_nbr27()
        assert np.array_equal(nb, oracle.neighbours(L)), f"nbr27 level {l}"
        if l > 0:
            assert np.array_equal(info.device_child8(), oracle.children(case.olv[l - 1], L)), f"child8 level {l}"
    # the finest level really is in the caller's order, and its lists are the sorted case's
    # lists with rows and entries renamed by the permutation
    assert np.array_equal(case.glv.info(0).device_coords(), case.coords)
    inv = np.empty_like(case.perm)
    inv[case.perm] = np.arange(case.perm.size)
    nb_sorted = case_batch64.glv.info(0).device_nbr27()[case.perm]
    assert np.array_equal(case.glv.info(0).device_nbr27(), np.where(nb_sorted >= 0, inv[np.maximum(nb_sorted, 0)], -1))


def test_neighbour_lists_with_short_sorted_runs(oracle):
    """Neighbouring lanes of the index-list kernel hand each other results when their voxels are
    z-neighbours.  Here every model's sorted voxel list is cut into runs of 1-7 voxels, the runs
    shuffled and every third one reversed: lanes with a z-neighbour above only, below only, on
    both sides and on neither sit side by side, also across wavefront and tile boundaries."""
    coords, offs, _ = S.config_batch(2)
    rng = np.random.default_rng(1618)
    pieces = []
    for v in range(len(offs) - 1):
        a, b = int(offs[v]), int(offs[v + 1])
        cuts = [a]
        while cuts[-1] < b:
            cuts.append(min(b, cuts[-1] + int(rng.integers(1, 8))))
        runs = [np.arange(cuts[q], cuts[q + 1]) for q in range(len(cuts) - 1)]
        runs = [r[::-1] if q % 3 == 2 else r for q, r in enumerate(runs)]
        pieces += [runs[q] for q in rng.permutation(len(runs))]
    perm = np.concatenate(pieces)
    assert np.array_equal(np.sort(perm), np.arange(coords.shape[0]))
    case = Case(oracle, np.ascontiguousarray(coords[perm]), offs, 64, 3)
    for l, L in enumerate(case.olv):
        info = case.glv.info(l)
        assert np.array_equal(info.device_coords(), L.coords)
        assert np.array_equal(info.device_nbr27(), oracle.neighbours(L)), f"nbr27 level {l}"
        if l > 0:
            assert np.array_equal(info.device_child8(), oracle.children(case.olv[l - 1], L)), f"child8 level {l}"


@pytest.mark.parametrize("algo", ALGOS, ids=ALGO_IDS)
@pytest.mark.parametrize("c_in,c_out", [(4, 32), (16, 4), (32, 64)])
def test_permuted_input_conv_and_pool(oracle, case_permuted, c_in, c_out, algo):
    case = case_permuted
    L = case.olv[0]
    n = L.Ntot
    X = S.normals_plus_one(case.normals) if c_in == 4 else S.gaussian((n, c_in), 1.0, 61)
    W = S.he_weights(c_in, c_out, 62)
    G = S.gaussian((n, c_out), 1.0, 63)
    Xp, Wp, Gp = oracle.to_paper_X(X), oracle.to_paper_W(W), oracle.to_paper_X(G)
    Y = _conv_fwd_gpu(case, 0, X, W, algo=algo)
    assert_close(Y, oracle.conv_fwd(L, Xp, Wp).T, what="fwd")
    ws = workspace(max(hch.hch_conv_workspace_bytes(case.glv, 0, c_in, c_out, hch.HCH_F32, k, algo)
                       for k in (hch.HCH_WS_BWD_DATA, hch.HCH_WS_BWD_WEIGHT)))
    dX = torch.full((n, c_in), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_conv_bwd_data(case.glv, 0, hch.HCH_F32, dev(G), dev(W), dX, c_in, c_out, ws, algo)
    assert_close(dX.cpu().numpy(), oracle.conv_bwd_data(L, Gp, Wp, c_in).T, what="bwd data")
    dW = torch.full((27, c_in, c_out), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_conv_bwd_weight(case.glv, 0, hch.HCH_F32, dev(X), dev(G), dW, c_in, c_out, ws, algo)
    assert_close(dW.cpu().numpy(), oracle.from_paper_W(oracle.conv_bwd_weight(L, Xp, Gp), c_in), what="bwd weight")
    # pooling of the GPU's own output from the permuted level to the (sorted) coarser one
    n1 = case.olv[1].Ntot
    P = torch.empty((n1, c_out), dtype=torch.float32, device="cuda")
    sw = torch.empty((n1, c_out), dtype=torch.int32, device="cuda")
    hch.hch_pool_fwd(case.glv, 0, dev(Y), P, sw, c_out)
    Po, swo = oracle.pool_max_fwd(L, case.olv[1], oracle.to_paper_X(Y))
    assert np.array_equal(sw.cpu().numpy(), swo.T) and np.array_equal(P.cpu().numpy(), Po.T.astype(np.float32))


# --------------------------------------------------------------------------------------
# pooling, ReLU
# --------------------------------------------------------------------------------------

@pytest.mark.parametrize("c", [1, 16, 37])
def test_pool_fwd_bwd(oracle, case_batch64, c):
    case = case_batch64
    lf, lc = case.olv[0], case.olv[1]
    X = S.gaussian((lf.Ntot, c), 1.0, 31)
    X[np.random.default_rng(32).random(X.shape) < 0.5] = 0.0        # ties, as after ReLU
    Y = torch.full((lc.Ntot, c), float("nan"), dtype=torch.float32, device="cuda")
    sw = torch.full((lc.Ntot, c), -7, dtype=torch.int32, device="cuda")
    hch.hch_pool_fwd(case.glv, 0, dev(X), Y, sw, c)
    Yo, swo = oracle.pool_max_fwd(lf, lc, oracle.to_paper_X(X))
    assert np.array_equal(sw.cpu().numpy(), swo.T)
    assert np.array_equal(Y.cpu().numpy(), Yo.T.astype(np.float32))
    dY = S.gaussian((lc.Ntot, c), 1.0, 33)
    dX = torch.full((lf.Ntot, c), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_pool_bwd(case.glv, 0, dev(dY), sw, dX, c)
    want = oracle.pool_max_bwd(lf.Ntot, oracle.to_paper_X(dY), swo).T
    assert np.array_equal(dX.cpu().numpy(), want.astype(np.float32))


@pytest.mark.parametrize("c", [1, 16, 37])
def test_fused_relu_pool(oracle, case_batch64, c):
    """ReLU + pool in one call, and pool backward + ReLU backward in one call, against the oracle's
    separate steps."""
    case = case_batch64
    lf, lc = case.olv[0], case.olv[1]
    Yin = S.gaussian((lf.Ntot, c), 1.0, 34)
    A = torch.full((lf.Ntot, c), float("nan"), dtype=torch.float32, device="cuda")
    P = torch.full((lc.Ntot, c), float("nan"), dtype=torch.float32, device="cuda")
    sw = torch.full((lc.Ntot, c), -7, dtype=torch.int32, device="cuda")
    hch.hch_relu_pool_fwd(case.glv, 0, dev(Yin), A, P, sw, c)
    Ao = np.maximum(Yin, 0)
    Po, swo = oracle.pool_max_fwd(lf, lc, oracle.to_paper_X(Ao))
    assert np.array_equal(A.cpu().numpy(), Ao)
    assert np.array_equal(sw.cpu().numpy(), swo.T)
    assert np.array_equal(P.cpu().numpy(), Po.T.astype(np.float32))
    dP = S.gaussian((lc.Ntot, c), 1.0, 35)
    dY = torch.full((lf.Ntot, c), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_pool_relu_bwd(case.glv, 0, dev(dP), sw, A, dY, c)
    dA = oracle.pool_max_bwd(lf.Ntot, oracle.to_paper_X(dP), swo).T
    assert np.array_equal(dY.cpu().numpy(), np.where(Ao > 0, dA, 0).astype(np.float32))
    # without storing the rectified rows: same pooled values and switches, and the backward
    # pass takes the sign from the values before the ReLU
    P2 = torch.full_like(P, float("nan"))
    sw2 = torch.full_like(sw, -7)
    hch.hch_relu_pool_fwd(case.glv, 0, dev(Yin), None, P2, sw2, c)
    assert torch.equal(P2, P) and torch.equal(sw2, sw)
    dY2 = torch.full_like(dY, float("nan"))
    hch.hch_pool_relu_bwd(case.glv, 0, dev(dP), sw2, dev(Yin), dY2, c)
    assert torch.equal(dY2, dY)
    # ... or from the pooled rows alone
    dY3 = torch.full_like(dY, float("nan"))
    hch.hch_pool_relu_bwd_pooled(case.glv, 0, dev(dP), sw2, P2, dY3, c)
    assert torch.equal(dY3, dY)


def test_relu():
    x = S.gaussian((100003,), 1.0, 41)
    y = torch.empty(x.size, dtype=torch.float32, device="cuda")
    hch.hch_relu_fwd(dev(x), y, x.size)
    assert np.array_equal(y.cpu().numpy(), np.maximum(x, 0))
    g = S.gaussian((100003,), 1.0, 42)
    dx = torch.empty_like(y)
    hch.hch_relu_bwd(y, dev(g), dx, x.size)
    assert np.array_equal(dx.cpu().numpy(), np.where(x > 0, g, 0).astype(np.float32))


# --------------------------------------------------------------------------------------
# errors
# --------------------------------------------------------------------------------------

def test_error_paths(case_sphere):
    case = case_sphere
    n = case.olv[0].Ntot
    X = dev(case.normals)
    W = dev(S.gaussian((27, 3, 16), 0.1, 0))
    Y = torch.empty((n, 16), dtype=torch.float32, device="cuda")
    with pytest.raises(hch.HchError) as ei:
        hch.hch_conv_fwd(case.glv, 0, hch.HCH_F32, X, W, Y, 3, 16, workspace(256))
    assert ei.value.status == 6
    with pytest.raises(hch.HchError) as ei:
        hch.hch_conv_fwd(case.glv, 5, hch.HCH_F32, X, W, Y, 3, 16, workspace(1 << 20))
    assert ei.value.status == 1
    with pytest.raises(hch.HchError) as ei:
        hch.hch_pool_fwd(case.glv, 1, X, Y, Y, 3)          # no coarser level below level 1
    assert ei.value.status == 1
    with pytest.raises(hch.HchError) as ei:
        hch.hch_hash2col(case.glv, 0, hch.HCH_F32, X, 3, n - 5, 10, Y)
    assert ei.value.status == 1
    n1 = case.olv[1].Ntot
    dP = torch.zeros((n1, 16), dtype=torch.float32, device="cuda")
    sw = torch.zeros((n1, 16), dtype=torch.int32, device="cuda")
    with pytest.raises(hch.HchError) as ei:
        hch.hch_pool_relu_bwd_pooled(case.glv, 1, dP, sw, dP, Y, 16)      # no coarser level below level 1
    assert ei.value.status == 1
    with pytest.raises(hch.HchError) as ei:
        hch.hch_pool_relu_bwd_pooled(case.glv, 0, dP, sw, dP[: n1 - 1], Y, 16)   # pooled rows one short
    assert ei.value.status == 1


def test_weight_gradient_from_resident_columns(case_small):
    """The weight gradient computed from the column matrix that the forward pass left in the
    workspace equals, bit for bit, the one that gathers the columns again; the option is
    refused by the other calls."""
    case = case_small
    n, ci, co = case.olv[0].Ntot, 16, 32
    F32, CO, RES = hch.HCH_F32, hch.HCH_ALGO_COLUMNS, hch.HCH_ALGO_COLUMNS_RESIDENT
    X, W, G = dev(S.gaussian((n, ci), 1.0, 61)), dev(S.gaussian((27, ci, co), 0.1, 62)), dev(S.gaussian((n, co), 1.0, 63))
    ws = workspace(max(hch.hch_conv_workspace_bytes(case.glv, 0, ci, co, F32, k, a)
                       for k in (hch.HCH_WS_FWD, hch.HCH_WS_BWD_WEIGHT) for a in (CO, RES)))
    Y = torch.empty((n, co), dtype=torch.float32, device="cuda")
    hch.hch_conv_fwd(case.glv, 0, F32, X, W, Y, ci, co, ws, CO)
    d1 = torch.full((27, ci, co), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_conv_bwd_weight(case.glv, 0, F32, X, G, d1, ci, co, ws, RES)
    d2 = torch.full((27, ci, co), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_conv_bwd_weight(case.glv, 0, F32, X, G, d2, ci, co, ws, CO)
    assert torch.equal(d1, d2)
    for fn, args in ((hch.hch_conv_fwd, (X, W, Y)), (hch.hch_conv_bwd_data, (G, W, torch.empty((n, ci), dtype=torch.float32, device="cuda")))):
        with pytest.raises(hch.HchError) as ei:
            fn(case.glv, 0, F32, *args, ci, co, ws, RES)
        assert ei.value.status == 1


# --------------------------------------------------------------------------------------
# bf16 inputs, fp32 accumulation
# --------------------------------------------------------------------------------------

TOL_BF16 = 2e-2     # stated bound for bf16-in / fp32-accumulate


def dev_bf16(a_on_grid):
    return dev(S.bf16_bits(a_on_grid).view(np.int16))


@pytest.fixture(scope="module")
def case_hires(oracle):
    # the high-resolution workload scaled down: two-voxel shells of 2..6 primitives
    coords, offs, _ = S.config_batch(5, batch=2, u=64)
    return Case(oracle, coords, offs, 64, 2)


@pytest.mark.parametrize("algo", ALGOS, ids=ALGO_IDS)
@pytest.mark.parametrize("c_in,c_out", [(64, 64), (8, 24), (6, 5), (16, 32), (32, 16), (24, 40), (128, 64), (64, 8)])
def test_conv_bf16(oracle, case_hires, c_in, c_out, algo):
    """X, W, dY are bf16 (both sides start from the same bf16-representable numbers); products
    are accumulated in fp32 on the GPU and in double in the oracle; outputs are fp32."""
    case = case_hires
    L = case.olv[0]
    n = L.Ntot
    X = S.to_bf16_grid(S.gaussian((n, c_in), 1.0, 51))
    W = S.to_bf16_grid(S.he_weights(c_in, c_out, 52))
    G = S.to_bf16_grid(S.gaussian((n, c_out), 1.0, 53))
    Xp, Wp, Gp = oracle.to_paper_X(X), oracle.to_paper_W(W), oracle.to_paper_X(G)
    B16 = hch.HCH_BF16

    def ws(kind):
        return workspace(hch.hch_conv_workspace_bytes(case.glv, 0, c_in, c_out, B16, kind, algo))

    Y = torch.full((n, c_out), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_conv_fwd(case.glv, 0, B16, dev_bf16(X), dev_bf16(W), Y, c_in, c_out, ws(hch.HCH_WS_FWD), algo)
    want = oracle.conv_fwd(L, Xp, Wp).T
    assert_close(Y.cpu().numpy(), want, tol=TOL_BF16, what="bf16 fwd")
    # exact products, fp32 sums: in fact as close as the fp32 path
    assert_close(Y.cpu().numpy(), want, tol=TOL_F32, what="bf16 fwd (fp32-level)")

    dX = torch.full((n, c_in), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_conv_bwd_data(case.glv, 0, B16, dev_bf16(G), dev_bf16(W), dX, c_in, c_out, ws(hch.HCH_WS_BWD_DATA), algo)
    assert_close(dX.cpu().numpy(), oracle.conv_bwd_data(L, Gp, Wp, c_in).T, tol=TOL_BF16, what="bf16 bwd data")

    dW = torch.full((27, c_in, c_out), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_conv_bwd_weight(case.glv, 0, B16, dev_bf16(X), dev_bf16(G), dW, c_in, c_out, ws(hch.HCH_WS_BWD_WEIGHT), algo)
    assert_close(dW.cpu().numpy(), oracle.from_paper_W(oracle.conv_bwd_weight(L, Xp, Gp), c_in), tol=TOL_BF16,
                 what="bf16 bwd weight")

    # with the tap-major copy of the index lists (another lay-out of the same indices): same bits
    tlv = hch.hch_build_levels(case.coords, case.offs, case.u, 1)
    hch.hch_build_tap_major(tlv, 0)
    hch.hch_build_neighbours(tlv, 0)          # a rebuild refreshes the copy
    for fn, a, b, ref, shape, kind in ((hch.hch_conv_fwd, X, W, Y, (n, c_out), hch.HCH_WS_FWD),
                                       (hch.hch_conv_bwd_data, G, W, dX, (n, c_in), hch.HCH_WS_BWD_DATA),
                                       (hch.hch_conv_bwd_weight, X, G, dW, (27, c_in, c_out), hch.HCH_WS_BWD_WEIGHT)):
        out = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
        fn(tlv, 0, B16, dev_bf16(a), dev_bf16(b), out, c_in, c_out, ws(kind), algo)
        assert torch.equal(out, ref), fn.__name__


# --------------------------------------------------------------------------------------
# degenerate and ragged cases
# --------------------------------------------------------------------------------------

@pytest.fixture(scope="module")
def case_tiny(oracle):
    """One-voxel models, a model in a grid corner and on the far faces (neighbours off the
    grid), a two-voxel model whose voxels touch only diagonally; 5 levels down to 1^3."""
    pts = [np.array([[7, 7, 7]]),
           np.array([[0, 0, 0], [1, 1, 1]]),
           np.array([[15, 15, 15], [15, 14, 15], [14, 15, 15], [15, 15, 14], [0, 15, 0]]),
           np.array([[3, 3, 3]])]
    coords = np.concatenate(pts).astype(np.int32)
    offs = np.cumsum([0] + [len(p) for p in pts])
    return Case(oracle, coords, offs, 16, 5)


@pytest.mark.parametrize("algo", ALGOS, ids=ALGO_IDS)
def test_tiny_models_all_levels(oracle, case_tiny, algo):
    case = case_tiny
    for l, L in enumerate(case.olv):
        info = case.glv.info(l)
        assert np.array_equal(info.device_nbr27(), oracle.neighbours(L))
        if l > 0:
            assert np.array_equal(info.device_child8(), oracle.children(case.olv[l - 1], L))
    for level, (c_in, c_out) in ((0, (1, 1)), (0, (4, 8)), (2, (2, 3)), (4, (8, 4))):
        L = case.olv[level]
        n = L.Ntot
        X = S.gaussian((n, c_in), 1.0, 61)
        W = S.gaussian((27, c_in, c_out), 0.3, 62)
        G = S.gaussian((n, c_out), 1.0, 63)
        Xp, Wp, Gp = oracle.to_paper_X(X), oracle.to_paper_W(W), oracle.to_paper_X(G)
        assert_close(_conv_fwd_gpu(case, level, X, W, algo=algo), oracle.conv_fwd(L, Xp, Wp).T, what="tiny fwd")
        ws = workspace(hch.hch_conv_workspace_bytes(case.glv, level, c_in, c_out, hch.HCH_F32, hch.HCH_WS_BWD_DATA, algo))
        dX = torch.full((n, c_in), float("nan"), dtype=torch.float32, device="cuda")
        hch.hch_conv_bwd_data(case.glv, level, hch.HCH_F32, dev(G), dev(W), dX, c_in, c_out, ws, algo)
        assert_close(dX.cpu().numpy(), oracle.conv_bwd_data(L, Gp, Wp, c_in).T, what="tiny bwd data")
        ws = workspace(hch.hch_conv_workspace_bytes(case.glv, level, c_in, c_out, hch.HCH_F32, hch.HCH_WS_BWD_WEIGHT, algo))
        dW = torch.full((27, c_in, c_out), float("nan"), dtype=torch.float32, device="cuda")
        hch.hch_conv_bwd_weight(case.glv, level, hch.HCH_F32, dev(X), dev(G), dW, c_in, c_out, ws, algo)
        assert_close(dW.cpu().numpy(), oracle.from_paper_W(oracle.conv_bwd_weight(L, Xp, Gp), c_in), what="tiny bwd weight")
    # pooling over every level pair
    for l in range(4):
        lf, lc = case.olv[l], case.olv[l + 1]
        X = S.gaussian((lf.Ntot, 3), 1.0, 64 + l)
        Y = torch.empty((lc.Ntot, 3), dtype=torch.float32, device="cuda")
        sw = torch.empty((lc.Ntot, 3), dtype=torch.int32, device="cuda")
        hch.hch_pool_fwd(case.glv, l, dev(X), Y, sw, 3)
        Yo, swo = oracle.pool_max_fwd(lf, lc, oracle.to_paper_X(X))
        assert np.array_equal(sw.cpu().numpy(), swo.T) and np.array_equal(Y.cpu().numpy(), Yo.T.astype(np.float32))


def test_pool_nan_and_negative_values(oracle, case_batch64):
    """Empty children never enter the maximum (all-negative inputs keep a negative maximum) and a
    NaN does not replace an earlier value."""
    case = case_batch64
    lf, lc = case.olv[0], case.olv[1]
    X = -np.abs(S.gaussian((lf.Ntot, 4), 1.0, 71)) - 0.5
    X[::97, 1] = np.nan
    Y = torch.empty((lc.Ntot, 4), dtype=torch.float32, device="cuda")
    sw = torch.empty((lc.Ntot, 4), dtype=torch.int32, device="cuda")
    hch.hch_pool_fwd(case.glv, 0, dev(X), Y, sw, 4)
    Yo, swo = oracle.pool_max_fwd(lf, lc, oracle.to_paper_X(X))
    assert np.array_equal(sw.cpu().numpy(), swo.T)
    got, want = Y.cpu().numpy(), Yo.T.astype(np.float32)
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.array_equal(got[~np.isnan(got)], want[~np.isnan(want)])
    assert (got[~np.isnan(got)] < 0).all()


# --------------------------------------------------------------------------------------
# transposed convolution and max-unpooling
# --------------------------------------------------------------------------------------

@pytest.mark.parametrize("algo", ALGOS, ids=ALGO_IDS)
@pytest.mark.parametrize("c_in,c_out,bf16", [(32, 16, False), (5, 3, False), (64, 32, True), (16, 64, True)])
def test_deconv(oracle, case_small, c_in, c_out, bf16, algo):
    case = case_small
    L = case.olv[1]
    n = L.Ntot
    X = S.gaussian((n, c_in), 1.0, 81)
    W = S.gaussian((27, c_out, c_in), 0.1, 82)         # forward conv c_out -> c_in, transposed here
    G = S.gaussian((n, c_out), 1.0, 83)
    if bf16:
        X, W, G = S.to_bf16_grid(X), S.to_bf16_grid(W), S.to_bf16_grid(G)
    Xp, Wp, Gp = oracle.to_paper_X(X), oracle.to_paper_W(W), oracle.to_paper_X(G)
    DT = hch.HCH_BF16 if bf16 else hch.HCH_F32
    put = (lambda a: dev(S.bf16_bits(a).view(np.int16))) if bf16 else dev
    tol = 2e-2 if bf16 else TOL_F32

    def ws(kind):
        return workspace(hch.hch_conv_workspace_bytes(case.glv, 1, c_out, c_in, DT, kind, algo))

    Y = torch.full((n, c_out), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_deconv_fwd(case.glv, 1, DT, put(X), put(W), Y, c_in, c_out, ws(hch.HCH_WS_BWD_DATA), algo)
    assert_close(Y.cpu().numpy(), oracle.deconv_fwd(L, Xp, Wp).T, tol=tol, what="deconv fwd")
    dX = torch.full((n, c_in), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_deconv_bwd_data(case.glv, 1, DT, put(G), put(W), dX, c_in, c_out, ws(hch.HCH_WS_FWD), algo)
    assert_close(dX.cpu().numpy(), oracle.conv_fwd(L, Gp, Wp).T, tol=tol, what="deconv bwd data")
    dW = torch.full((27, c_out, c_in), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_deconv_bwd_weight(case.glv, 1, DT, put(X), put(G), dW, c_in, c_out, ws(hch.HCH_WS_BWD_WEIGHT), algo)
    assert_close(dW.cpu().numpy(), oracle.from_paper_W(oracle.conv_bwd_weight(L, Gp, Xp), c_out), tol=tol, what="deconv bwd weight")


def test_unpool(oracle, case_batch64):
    case = case_batch64
    lf, lc = case.olv[0], case.olv[1]
    c = 6
    X = S.gaussian((lf.Ntot, c), 1.0, 84)
    P = torch.empty((lc.Ntot, c), dtype=torch.float32, device="cuda")
    sw = torch.empty((lc.Ntot, c), dtype=torch.int32, device="cuda")
    hch.hch_pool_fwd(case.glv, 0, dev(X), P, sw, c)
    U = torch.full((lf.Ntot, c), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_unpool_fwd(case.glv, 0, P, sw, U, c)
    Po, swo = oracle.pool_max_fwd(lf, lc, oracle.to_paper_X(X))
    assert np.array_equal(U.cpu().numpy(), oracle.unpool_max_fwd(lf.Ntot, Po, swo).T.astype(np.float32))
    G = S.gaussian((lf.Ntot, c), 1.0, 85)
    dP = torch.full((lc.Ntot, c), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_unpool_bwd(case.glv, 0, dev(G), sw, dP, c)
    assert np.array_equal(dP.cpu().numpy(), oracle.unpool_max_bwd(oracle.to_paper_X(G), swo).T.astype(np.float32))


# --------------------------------------------------------------------------------------
# tables constructed on the device: valid, and every lookup through them is the same
# --------------------------------------------------------------------------------------

def _check_device_built(oracle, olv, dlv):
    for l, L in enumerate(olv):
        info = dlv.info(l)
        assert info.n_total == L.Ntot
        assert np.array_equal(info.mbar, L.mbar), "hash table sides are fixed by n (Section 5.2)"
        assert np.array_equal(info.M, L.M) and np.array_equal(info.N, L.N)
        H, T, Phi, V = info.device_H(), info.device_T(), info.device_Phi(), info.device_V()
        assert np.array_equal(info.H_host(), H) and np.array_equal(info.T_host(), T)
        assert np.array_equal(info.Phi_host(), Phi)
        coords = info.device_coords()
        assert np.array_equal(coords, L.coords)
        R = np.asarray(info.R)
        for v in range(L.b):
            n = int(L.N[v + 1] - L.N[v]); m = int(info.mbar[v]); r = int(info.rbar[v])
            assert int(R[v + 1] - R[v]) == r ** 3 and np.gcd(r, m) == 1
            h = H[L.M[v]:L.M[v + 1]]
            occ = h >= 0
            # a perfect hash: every data index exactly once, the other slots empty
            assert int(occ.sum()) == n and np.array_equal(np.sort(h[occ]), np.arange(n))
            assert np.all(h[~occ] == -1)
            t = T[L.M[v]:L.M[v + 1]]
            assert np.array_equal(t[occ].astype(np.int64), coords[L.N[v]:L.N[v + 1]][h[occ]])
            assert np.all(t[~occ] == 0xFFFF)
            assert np.all(V[L.M[v]:L.M[v + 1]] == v)
            ph = Phi[R[v]:R[v + 1]].astype(np.int64)
            assert ph.max(initial=0) < m
            # Eq.1 with these tables sends every voxel to the slot that holds it
            p = coords[L.N[v]:L.N[v + 1]].astype(np.int64)
            cell = ((p[:, 0] % r) * r + p[:, 1] % r) * r + p[:, 2] % r
            s = (p % m + ph[cell]) % m
            slot = (s[:, 0] * m + s[:, 1]) * m + s[:, 2]
            assert np.array_equal(h[slot], np.arange(n))
        # lookups: occupied positions found, empty ones null, for all 27 / 8 probes of every voxel
        assert np.array_equal(info.device_nbr27(), oracle.neighbours(L)), f"nbr27 level {l}"
        if l > 0:
            assert np.array_equal(info.device_child8(), oracle.children(olv[l - 1], L)), f"child8 level {l}"


@pytest.mark.parametrize("name", ["case_sphere", "case_batch64", "case_small"])
def test_device_built_tables(request, oracle, name):
    case = request.getfixturevalue(name)
    dlv = hch.hch_build_levels_device(case.coords, case.offs, case.u, len(case.olv))
    torch.cuda.synchronize()
    _check_device_built(oracle, case.olv, dlv)
    # a convolution through them gives the same bits as through the host-built tables
    L = case.olv[0]
    X = S.gaussian((L.Ntot, 8), 1.0, 71)
    W = S.gaussian((27, 8, 16), 0.1, 72)
    outs = []
    for lv in (case.glv, dlv):
        Y = torch.full((L.Ntot, 16), float("nan"), dtype=torch.float32, device="cuda")
        ws = workspace(hch.hch_conv_workspace_bytes(lv, 0, 8, 16, hch.HCH_F32, hch.HCH_WS_FWD, hch.HCH_ALGO_FUSED))
        hch.hch_conv_fwd(lv, 0, hch.HCH_F32, dev(X), dev(W), Y, 8, 16, ws, hch.HCH_ALGO_FUSED)
        outs.append(Y)
    assert torch.equal(outs[0], outs[1])


def test_device_build_tiny_and_errors():
    # one voxel per model, a full 2^3 block, and the argument checks of the host entry point
    coords = np.array([[0, 0, 0], [3, 3, 3]] + [[x, y, z] for x in (0, 1) for y in (0, 1) for z in (0, 1)], np.int32)
    offs = np.array([0, 1, 2, 10], np.int64)
    dlv = hch.hch_build_levels_device(coords, offs, 4, 3)
    hlv = hch.hch_build_levels(coords, offs, 4, 3)
    torch.cuda.synchronize()
    for l in range(3):
        a, b = dlv.info(l), hlv.info(l)
        assert np.array_equal(a.device_nbr27(), b.device_nbr27())
        if l > 0:
            assert np.array_equal(a.device_child8(), b.device_child8())
    with pytest.raises(hch.HchError):
        hch.hch_build_levels_device(np.array([[0, 0, 0], [0, 0, 0]], np.int32), np.array([0, 2], np.int64), 4, 1)
    with pytest.raises(hch.HchError):
        hch.hch_build_levels_device(np.array([[0, 0, 5]], np.int32), np.array([0, 1], np.int64), 4, 1)


# --------------------------------------------------------------------------------------
# general kernel side / stride / padding across two levels, average pooling
# --------------------------------------------------------------------------------------

@pytest.mark.parametrize("F,stride,pad", [(3, 1, 1), (5, 1, 2), (3, 2, 1), (2, 2, 0), (4, 2, 1), (3, 4, 1)])
def test_field_lists_bit_exact(oracle, case_batch64, F, stride, pad):
    case = case_batch64
    shift = {1: 0, 2: 1, 4: 2}[stride]
    Li, Lo = case.olv[0], case.olv[shift]
    field = torch.full((Lo.Ntot, F ** 3), -7, dtype=torch.int32, device="cuda")
    field_t = torch.full((Li.Ntot, F ** 3), -7, dtype=torch.int32, device="cuda")
    hch.hch_field_build(case.glv, 0, F, stride, pad, field, field_t)
    want = oracle.field_indices(Li, Lo, F, stride, pad)
    got = field.cpu().numpy()
    assert np.array_equal(got, want)
    # the transposed rows are the inverse relation: field_t[i][row] = o  <=>  field[o][row] = i
    want_t = np.full((Li.Ntot, F ** 3), -1, np.int32)
    o, row = np.nonzero(want >= 0)
    want_t[want[o, row], row] = o
    assert np.array_equal(field_t.cpu().numpy(), want_t)
    if F == 3 and stride == 1:
        assert np.array_equal(got, case.glv.info(0).device_nbr27())


@pytest.mark.parametrize("F,stride,pad,c_in,c_out,bf16", [
    (3, 2, 1, 8, 16, False), (2, 2, 0, 4, 8, False), (5, 1, 2, 4, 8, False), (3, 2, 1, 3, 5, False), (3, 4, 1, 8, 8, False),
    (3, 2, 1, 16, 32, True), (2, 2, 0, 64, 64, True), (5, 1, 2, 8, 8, True), (3, 2, 1, 6, 5, True)])
def test_general_conv(oracle, case_small, F, stride, pad, c_in, c_out, bf16):
    """Forward, weight gradient and data gradient of a strided / larger convolution between two
    levels against the oracle's Algorithm 1 / 2, in fp32 and with bf16 inputs."""
    case = case_small
    shift = {1: 0, 2: 1, 4: 2}[stride]
    Li, Lo = case.olv[0], case.olv[shift]
    F3 = F ** 3
    X = S.gaussian((Li.Ntot, c_in), 1.0, 101)
    W = S.gaussian((F3, c_in, c_out), 0.1, 102)
    G = S.gaussian((Lo.Ntot, c_out), 1.0, 103)
    if bf16:
        X, W, G = S.to_bf16_grid(X), S.to_bf16_grid(W), S.to_bf16_grid(G)
    put = dev_bf16 if bf16 else dev
    tol = TOL_BF16 if bf16 else TOL_F32
    field = torch.empty((Lo.Ntot, F3), dtype=torch.int32, device="cuda")
    field_t = torch.empty((Li.Ntot, F3), dtype=torch.int32, device="cuda")
    hch.hch_field_build(case.glv, 0, F, stride, pad, field, field_t)
    DT = hch.HCH_BF16 if bf16 else hch.HCH_F32
    ws = workspace(max(hch.hch_sconv_workspace_bytes(case.glv, 0, F, stride, c_in, c_out, DT, k)
                       for k in (hch.HCH_WS_FWD, hch.HCH_WS_BWD_DATA, hch.HCH_WS_BWD_WEIGHT)))
    Xp, Wp, Gp = oracle.to_paper_X(X), oracle.to_paper_W(W), oracle.to_paper_X(G)
    Y = torch.full((Lo.Ntot, c_out), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_sconv_fwd(case.glv, 0, F, stride, DT, put(X), put(W), Y, field, c_in, c_out, ws)
    assert_close(Y.cpu().numpy(), oracle.sconv_fwd(Li, Lo, Xp, Wp, F, stride, pad).T, tol=tol, what="general fwd")
    dW = torch.full((F3, c_in, c_out), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_sconv_bwd_weight(case.glv, 0, F, stride, DT, put(X), put(G), dW, field, c_in, c_out, ws)
    want_dW = oracle.sconv_bwd_weight(Li, Lo, Xp, Gp, F, stride, pad).reshape(c_out, c_in, F3).transpose(2, 1, 0)
    assert_close(dW.cpu().numpy(), want_dW, tol=tol, what="general bwd weight")
    dX = torch.full((Li.Ntot, c_in), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_sconv_bwd_data(case.glv, 0, F, stride, DT, put(G), put(W), dX, field_t, c_in, c_out, ws)
    assert_close(dX.cpu().numpy(), oracle.sconv_bwd_data(Li, Lo, Gp, Wp, c_in, F, stride, pad).T, tol=tol, what="general bwd data")


def test_general_conv_equals_3x3x3(case_small):
    """F = 3, stride 1 through the general entry points gives the bits of hch_conv_fwd with the fused
    algorithm that multiplies every tap (HCH_ALGO_FUSED_DENSE); the default fused algorithm leaves
    out the taps a tile of voxels lacks, which changes where a split reduction is cut and hence
    the rounding, not the sums."""
    case = case_small
    n = case.olv[0].Ntot
    X, W = dev(S.gaussian((n, 32), 1.0, 111)), dev(S.gaussian((27, 32, 64), 0.1, 112))
    field = torch.empty((n, 27), dtype=torch.int32, device="cuda")
    hch.hch_field_build(case.glv, 0, 3, 1, 1, field, None)
    F32, FU, FD = hch.HCH_F32, hch.HCH_ALGO_FUSED, hch.HCH_ALGO_FUSED_DENSE
    Y1 = torch.empty((n, 64), dtype=torch.float32, device="cuda")
    Y2, Y3 = torch.empty_like(Y1), torch.empty_like(Y1)
    hch.hch_sconv_fwd(case.glv, 0, 3, 1, F32, X, W, Y1, field, 32, 64,
                      workspace(hch.hch_sconv_workspace_bytes(case.glv, 0, 3, 1, 32, 64, F32, hch.HCH_WS_FWD)))
    hch.hch_conv_fwd(case.glv, 0, F32, X, W, Y2, 32, 64,
                     workspace(hch.hch_conv_workspace_bytes(case.glv, 0, 32, 64, F32, hch.HCH_WS_FWD, FD)), FD)
    assert torch.equal(Y1, Y2)
    hch.hch_conv_fwd(case.glv, 0, F32, X, W, Y3, 32, 64,
                     workspace(hch.hch_conv_workspace_bytes(case.glv, 0, 32, 64, F32, hch.HCH_WS_FWD, FU)), FU)
    assert_close(Y3.cpu().numpy(), Y2.cpu().numpy(), what="fused vs fused without tap skipping")


@pytest.mark.parametrize("c", [1, 16, 37])
def test_avgpool(oracle, case_batch64, c):
    case = case_batch64
    lf, lc = case.olv[0], case.olv[1]
    X = S.gaussian((lf.Ntot, c), 1.0, 121)
    G = S.gaussian((lc.Ntot, c), 1.0, 122)
    Y = torch.full((lc.Ntot, c), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_avgpool_fwd(case.glv, 0, dev(X), Y, c)
    assert_close(Y.cpu().numpy(), oracle.avgpool_fwd(lf, lc, oracle.to_paper_X(X)).T, what="avgpool fwd")
    dX = torch.full((lf.Ntot, c), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_avgpool_bwd(case.glv, 0, dev(G), dX, c)
    want = oracle.avgpool_bwd(lf, lc, oracle.to_paper_X(G)).T
    assert np.array_equal(dX.cpu().numpy(), want.astype(np.float32))      # one exact scaling per element


def test_general_conv_errors(case_batch64):
    case = case_batch64
    n = case.olv[0].Ntot
    f = torch.empty((n, 27), dtype=torch.int32, device="cuda")
    for F, stride, pad, level in ((4, 1, 1, 0), (3, 3, 1, 0), (3, 1, 0, 0), (3, 2, 3, 0), (3, 2, 1, 2), (8, 2, 1, 0)):
        with pytest.raises(hch.HchError):
            hch.hch_field_build(case.glv, level, F, stride, pad, f, None)
    with pytest.raises(hch.HchError):
        hch.hch_field_build(case.glv, 0, 3, 1, 1, None, None)


# --------------------------------------------------------------------------------------
# the two forms of the products' main loop: same tiles, same order of sums, same bits
# --------------------------------------------------------------------------------------

@pytest.mark.parametrize("algo", [hch.HCH_ALGO_COLUMNS, hch.HCH_ALGO_FUSED, hch.HCH_ALGO_FUSED_DENSE],
                         ids=["columns", "fused", "fused-dense"])
@pytest.mark.parametrize("c_in,c_out,bf16", [(64, 128, False), (64, 128, True), (16, 32, False), (32, 16, False)],
                         ids=["f32-64-128", "bf16-64-128", "f32-16-32", "f32-32-16"])
def test_lean_and_pointer_loops_agree_bit_for_bit(case_small, algo, c_in, c_out, bf16):
    """hch_set_lean_loops(0) sends every product through the pointer-based loop; with channel
    counts that qualify for the lean loop (rows of a multiple of 32 channels, of 16 for the
    forward product's 16-wide tiles, of 64 with bf16) the outputs must not change by a bit.
    Both levels: the finest has enough voxels for the wide tiles, the next is split along the
    reduction."""
    case = case_small
    DT = hch.HCH_BF16 if bf16 else hch.HCH_F32
    put = (lambda a: dev(S.bf16_bits(S.to_bf16_grid(a)).view(np.int16))) if bf16 else dev
    for level in (0, 1):
        n = case.olv[level].Ntot
        X, G = put(S.gaussian((n, c_in), 1.0, 901 + level)), put(S.gaussian((n, c_out), 1.0, 903 + level))
        W = put(S.gaussian((27, c_in, c_out), 0.1, 905 + level))

        def ws(kind):
            return workspace(hch.hch_conv_workspace_bytes(case.glv, level, c_in, c_out, DT, kind, algo))

        outs = []
        try:
            for lean in (1, 0):
                hch.hch_set_lean_loops(lean)
                Y = torch.full((n, c_out), float("nan"), dtype=torch.float32, device="cuda")
                dX = torch.full((n, c_in), float("nan"), dtype=torch.float32, device="cuda")
                dW = torch.full((27, c_in, c_out), float("nan"), dtype=torch.float32, device="cuda")
                hch.hch_conv_fwd(case.glv, level, DT, X, W, Y, c_in, c_out, ws(hch.HCH_WS_FWD), algo)
                hch.hch_conv_bwd_data(case.glv, level, DT, G, W, dX, c_in, c_out, ws(hch.HCH_WS_BWD_DATA), algo)
                hch.hch_conv_bwd_weight(case.glv, level, DT, X, G, dW, c_in, c_out, ws(hch.HCH_WS_BWD_WEIGHT), algo)
                torch.cuda.synchronize()
                outs.append((Y, dX, dW))
        finally:
            assert hch.hch_set_lean_loops(1) == 0
        for a, b, what in zip(outs[0], outs[1], ("Y", "dX", "dW")):
            assert not torch.isnan(a).any(), what
            assert torch.equal(a, b), f"level {level} {what}: lean and pointer-based loops differ"
