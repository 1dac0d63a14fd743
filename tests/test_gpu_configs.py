"""GPU parity at the full size of the two workloads that are not the benchmark's: the backward
pass of a 32 -> 64 convolution on a 128^3 grid, batch 16, and the bf16 64 -> 64 convolution
forward and backward on a 512^3 grid, batch 4, with the tables of 5 levels.  Tables and index
lists are compared in full (bit-exact) and so is every floating-point output.

128^3: the oracle's column matrix is 279 722 x 864 doubles = 1.9 GB, so its hash2col -> product
-> col2hash (Eq.7, Eq.8) gives every element of dX and dW directly.

512^3: the column matrix of the whole batch would be 2 976 869 x 1728 doubles = 41 GB.  Y and dX
are therefore evaluated voxel by voxel from the definitions (Eq.2, Eq.8) for ALL voxels, in
blocks; dW (Eq.7) is a sum over the voxels and no lookup crosses models, so it is the sum of
the oracle's hash2col^T . dY over one model at a time (about 10 GB each)."""
import numpy as np
import pytest

import synth_shapes as S

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
hch = pytest.importorskip("paper_1803_11385_amd")

TOL_F32 = 1e-4
TOL_BF16 = 2e-2
ALGOS = [hch.HCH_ALGO_FUSED, hch.HCH_ALGO_COLUMNS]
ALGO_IDS = ["fused", "columns"]


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda")


def dev_bf16(a_on_grid):
    return dev(S.bf16_bits(a_on_grid).view(np.int16))


def close(got, want, what, tol):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    rms = float(np.sqrt((want ** 2).mean()))
    err = np.abs(got - want)
    worst = float((err / (tol * (np.abs(want) + rms))).max())
    assert np.isfinite(got).all() and worst <= 1.0, f"{what}: err/bound {worst:.3g}, max abs {err.max():.3g}, rms {rms:.3g}"


def workspace(nbytes):
    # every byte 0xFF (NaN as a float, -1 as an index): a read of something the library did not write shows
    t = torch.full((int(nbytes) + 256,), 255, dtype=torch.uint8, device="cuda")
    off = (-t.data_ptr()) % 256
    return t[off: off + int(nbytes)]


def check_tables(oracle, olv, glv):
    for l, L in enumerate(olv):
        info = glv.info(l)
        assert info.n_total == L.Ntot
        assert np.array_equal(info.device_H(), L.H) and np.array_equal(info.device_T(), L.T)
        assert np.array_equal(info.device_Phi(), L.Phi) and np.array_equal(info.device_V(), L.V)
        assert np.array_equal(info.M, L.M) and np.array_equal(info.R, L.R) and np.array_equal(info.N, L.N)
        assert np.array_equal(info.device_nbr27(), oracle.neighbours(L)), f"nbr27 level {l}"
        if l > 0:
            assert np.array_equal(info.device_child8(), oracle.children(olv[l - 1], L)), f"child8 level {l}"


# --------------------------------------------------------------------------------------
# 128^3, batch 16: backward of 32 -> 64, fp32
# --------------------------------------------------------------------------------------

@pytest.fixture(scope="module")
def backward128(oracle):
    coords, offs, _ = S.config_batch(3)
    olv = oracle.build_hierarchy(coords, offs, 128, 1)
    glv = hch.hch_build_levels(coords, offs, 128, 1)
    n = olv[0].Ntot
    d = dict(olv=olv, glv=glv, X=S.gaussian((n, 32), 1.0, 3001), W=S.he_weights(32, 64, 3002),
             G=S.gaussian((n, 64), 1.0, 3003))
    Gp, Wp, Xp = oracle.to_paper_X(d["G"]), oracle.to_paper_W(d["W"]), oracle.to_paper_X(d["X"])
    d["want_dX"] = oracle.conv_bwd_data(olv[0], Gp, Wp, 32).T
    d["want_dW"] = oracle.from_paper_W(oracle.conv_bwd_weight(olv[0], Xp, Gp), 32)
    return d


def test_backward128_tables(oracle, backward128):
    check_tables(oracle, backward128["olv"], backward128["glv"])


@pytest.mark.parametrize("algo", ALGOS, ids=ALGO_IDS)
def test_backward128_gradients(oracle, backward128, algo):
    """dX through the data-gradient product and col2hash (or their fused form), dW = col^T dY:
    every element against the oracle."""
    d = backward128
    L, glv = d["olv"][0], d["glv"]
    n, ci, co = L.Ntot, 32, 64
    F32 = hch.HCH_F32
    X, W, G = dev(d["X"]), dev(d["W"]), dev(d["G"])
    dX = torch.full((n, ci), float("nan"), dtype=torch.float32, device="cuda")
    dW = torch.full((27, ci, co), float("nan"), dtype=torch.float32, device="cuda")
    ws = workspace(max(hch.hch_conv_workspace_bytes(glv, 0, ci, co, F32, k, algo)
                       for k in (hch.HCH_WS_BWD_DATA, hch.HCH_WS_BWD_WEIGHT)))
    hch.hch_conv_bwd_data(glv, 0, F32, G, W, dX, ci, co, ws, algo)
    hch.hch_conv_bwd_weight(glv, 0, F32, X, G, dW, ci, co, ws, algo)
    torch.cuda.synchronize()
    close(dX.cpu().numpy(), d["want_dX"], "dX", TOL_F32)
    close(dW.cpu().numpy(), d["want_dW"], "dW", TOL_F32)


# --------------------------------------------------------------------------------------
# 512^3, batch 4: 64 -> 64 with bf16 inputs
# --------------------------------------------------------------------------------------

@pytest.fixture(scope="module")
def hires512(oracle):
    coords, offs, _ = S.config_batch(5)
    olv = oracle.build_hierarchy(coords, offs, 512, 5)
    glv = hch.hch_build_levels(coords, offs, 512, 5)
    n = olv[0].Ntot
    print(f"512^3 batch 4: N per level = {[L.Ntot for L in olv]}", flush=True)
    d = dict(coords=coords, offs=np.asarray(offs, np.int64), olv=olv, glv=glv,
             X=S.to_bf16_grid(S.gaussian((n, 64), 1.0, 5001)),
             W=S.to_bf16_grid(S.he_weights(64, 64, 5002)), G=S.to_bf16_grid(S.gaussian((n, 64), 1.0, 5003)))
    d["Xd"], d["Wd"], d["Gd"] = dev_bf16(d["X"]), dev_bf16(d["W"]), dev_bf16(d["G"])
    return d


def _all_voxels(fn, n, block=1 << 18):
    return np.concatenate([fn(np.arange(a, min(n, a + block), dtype=np.int64)) for a in range(0, n, block)])


@pytest.fixture(scope="module")
def want_Y512(oracle, hires512):
    d = hires512
    L = d["olv"][0]
    Xp, Wp = oracle.to_paper_X(d["X"]), oracle.to_paper_W(d["W"])
    return _all_voxels(lambda idx: oracle.conv_fwd_at(L, Xp, Wp, idx), L.Ntot)


@pytest.fixture(scope="module")
def want_dX512(oracle, hires512):
    d = hires512
    L = d["olv"][0]
    Gp, Wp = oracle.to_paper_X(d["G"]), oracle.to_paper_W(d["W"])
    return _all_voxels(lambda idx: oracle.conv_bwd_data_at(L, Gp, Wp, 64, idx), L.Ntot)


@pytest.fixture(scope="module")
def want_dW512(oracle, hires512):
    d = hires512
    offs, total = d["offs"], np.zeros((64, 64 * 27), np.float64)
    for v in range(len(offs) - 1):
        a, b = int(offs[v]), int(offs[v + 1])
        Lv = oracle.build_hierarchy(d["coords"][a:b], [0, b - a], 512, 1)[0]
        total += oracle.conv_bwd_weight(Lv, oracle.to_paper_X(d["X"][a:b]), oracle.to_paper_X(d["G"][a:b]))
    return oracle.from_paper_W(total, 64)


def test_hires512_tables(oracle, hires512):
    check_tables(oracle, hires512["olv"], hires512["glv"])


def _fused_ws(glv, B16):
    return workspace(max(hch.hch_conv_workspace_bytes(glv, 0, 64, 64, B16, k, hch.HCH_ALGO_FUSED)
                         for k in (hch.HCH_WS_FWD, hch.HCH_WS_BWD_DATA, hch.HCH_WS_BWD_WEIGHT)))


def test_hires512_bf16_forward(oracle, hires512, want_Y512):
    """bf16 inputs, fp32 accumulation: forward with both algorithms (the columns one with a
    workspace that holds only part of the column matrix, so that it runs in chunks); every
    element of Y."""
    d = hires512
    glv, n, ci, co, B16 = d["glv"], d["olv"][0].Ntot, 64, 64, hch.HCH_BF16
    FU, CO = hch.HCH_ALGO_FUSED, hch.HCH_ALGO_COLUMNS
    Y = torch.full((n, co), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_conv_fwd(glv, 0, B16, d["Xd"], d["Wd"], Y, ci, co, _fused_ws(glv, B16), FU)
    close(Y.cpu().numpy(), want_Y512, "fwd fused", TOL_BF16)
    # a quarter of the column matrix (n * 27 * 64 bf16 elements in all)
    part = workspace(hch.hch_conv_workspace_bytes(glv, 0, ci, co, B16, hch.HCH_WS_MIN, CO) + (n // 4) * 27 * ci * 2)
    Y.fill_(float("nan"))
    hch.hch_conv_fwd(glv, 0, B16, d["Xd"], d["Wd"], Y, ci, co, part, CO)
    close(Y.cpu().numpy(), want_Y512, "fwd columns, chunked", TOL_BF16)


@pytest.mark.parametrize("algo", ALGOS, ids=ALGO_IDS)
def test_hires512_bf16_data_gradient(oracle, hires512, want_dX512, algo):
    d = hires512
    glv, n, ci, co, B16 = d["glv"], d["olv"][0].Ntot, 64, 64, hch.HCH_BF16
    ws = workspace(hch.hch_conv_workspace_bytes(glv, 0, ci, co, B16, hch.HCH_WS_BWD_DATA, algo))
    dX = torch.full((n, ci), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_conv_bwd_data(glv, 0, B16, d["Gd"], d["Wd"], dX, ci, co, ws, algo)
    close(dX.cpu().numpy(), want_dX512, "dX", TOL_BF16)


@pytest.mark.parametrize("algo", ALGOS, ids=ALGO_IDS)
def test_hires512_bf16_weight_gradient(oracle, hires512, want_dW512, algo):
    d = hires512
    glv, ci, co, B16 = d["glv"], 64, 64, hch.HCH_BF16
    ws = workspace(hch.hch_conv_workspace_bytes(glv, 0, ci, co, B16, hch.HCH_WS_BWD_WEIGHT, algo))
    dW = torch.full((27, ci, co), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_conv_bwd_weight(glv, 0, B16, d["Xd"], d["Gd"], dW, ci, co, ws, algo)
    close(dW.cpu().numpy(), want_dW512, "dW", TOL_BF16)


def test_hires512_bf16_tap_major_indices(oracle, hires512, want_Y512, want_dX512, want_dW512):
    """The three fused products again after hch_build_tap_major: the tap-major copy of the index
    rows must not change a bit of the results (and they are checked against the oracle again).
    Runs last in this module: the copy stays with the level set."""
    d = hires512
    glv, n, ci, co, B16, FU = d["glv"], d["olv"][0].Ntot, 64, 64, hch.HCH_BF16, hch.HCH_ALGO_FUSED
    ws = _fused_ws(glv, B16)

    def run():
        Y = torch.full((n, co), float("nan"), dtype=torch.float32, device="cuda")
        dX = torch.full((n, ci), float("nan"), dtype=torch.float32, device="cuda")
        dW = torch.full((27, ci, co), float("nan"), dtype=torch.float32, device="cuda")
        hch.hch_conv_fwd(glv, 0, B16, d["Xd"], d["Wd"], Y, ci, co, ws, FU)
        hch.hch_conv_bwd_data(glv, 0, B16, d["Gd"], d["Wd"], dX, ci, co, ws, FU)
        hch.hch_conv_bwd_weight(glv, 0, B16, d["Xd"], d["Gd"], dW, ci, co, ws, FU)
        torch.cuda.synchronize()
        return Y.cpu().numpy(), dX.cpu().numpy(), dW.cpu().numpy()

    before = run()
    hch.hch_build_tap_major(glv, 0)
    after = run()
    for a, b, what in zip(before, after, ("Y", "dX", "dW")):
        assert np.array_equal(a, b), f"{what} changed with the tap-major index copy"
    close(after[0], want_Y512, "fwd", TOL_BF16)
    close(after[1], want_dX512, "dX", TOL_BF16)
    close(after[2], want_dW512, "dW", TOL_BF16)
