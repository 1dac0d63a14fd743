"""GPU parity for level sets whose resolutions are in ratios other than 2 (Section 4: a PSH can
be generated on a grid of any resolution, which allows any stride): tables and index lists
bit-exact (host-built) or valid with identical lookups (device-built), strided convolutions
and pooling between such levels against the oracle's Algorithm 1 / 2 traversal."""
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
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    assert got.shape == want.shape and np.isfinite(got).all(), what
    rms = float(np.sqrt((want ** 2).mean())) if want.size else 0.0
    err = np.abs(got - want)
    worst = float((err / np.maximum(tol * (np.abs(want) + rms), 1e-300)).max()) if want.size else 0.0
    assert worst <= 1.0, f"{what}: max err/bound = {worst:.3g}, max abs err = {err.max():.3g}"


def workspace(nbytes):
    # every byte 0xFF (NaN as a float, -1 as an index): a read of something the library did not write shows
    t = torch.full((max(nbytes, 256) + 256,), 255, dtype=torch.uint8, device="cuda")
    off = (-t.data_ptr()) % 256
    return t[off: off + max(nbytes, 256)]


# (finest side, ratios): 48 -> 16 -> 8, and sides the ratios do not divide: 50 -> 17 -> 9, 35 -> 7
SETS = [(48, (3, 2)), (50, (3, 2)), (35, (5,))]


@pytest.fixture(scope="module", params=SETS, ids=lambda p: f"{p[0]}:{'x'.join(map(str, p[1]))}")
def ratio_case(request, oracle):
    u, ratios = request.param
    coords, offs, _ = S.config_batch(2, batch=3, u=u)
    olv = oracle.build_hierarchy(coords, offs, u, len(ratios) + 1, ratios=list(ratios))
    glv = hch.hch_build_levels_ratios(coords, offs, u, ratios)
    torch.cuda.synchronize()
    return dict(u=u, ratios=ratios, coords=coords, offs=offs, olv=olv, glv=glv)


def test_ratio_tables_bit_exact(oracle, ratio_case):
    d = ratio_case
    for l, L in enumerate(d["olv"]):
        info = d["glv"].info(l)
        assert info.ubar == L.ubar
        assert np.array_equal(info.mbar, L.mbar) and np.array_equal(info.rbar, L.rbar)
        assert np.array_equal(info.M, L.M) and np.array_equal(info.R, L.R) and np.array_equal(info.N, L.N)
        assert np.array_equal(info.device_H(), L.H) and np.array_equal(info.device_T(), L.T)
        assert np.array_equal(info.device_Phi(), L.Phi) and np.array_equal(info.device_V(), L.V)
        assert np.array_equal(info.device_coords(), L.coords)
        assert np.array_equal(info.device_nbr27(), oracle.neighbours(L)), f"nbr27 level {l}"
        if l > 0 and d["ratios"][l - 1] == 2:
            assert np.array_equal(info.device_child8(), oracle.children(d["olv"][l - 1], L)), f"child8 level {l}"


def test_ratio_tables_built_on_device(oracle, ratio_case):
    d = ratio_case
    dlv = hch.hch_build_levels_ratios(d["coords"], d["offs"], d["u"], d["ratios"], device_tables=True)
    torch.cuda.synchronize()
    for l, L in enumerate(d["olv"]):
        info = dlv.info(l)
        assert info.ubar == L.ubar and info.n_total == L.Ntot
        assert np.array_equal(info.mbar, L.mbar) and np.array_equal(info.N, L.N)
        assert np.array_equal(info.device_coords(), L.coords)
        H = info.device_H()
        for v in range(L.b):
            h = H[L.M[v]:L.M[v + 1]]
            n = int(L.N[v + 1] - L.N[v])
            assert np.array_equal(np.sort(h[h >= 0]), np.arange(n))
        # every lookup through the device-built tables is the same
        assert np.array_equal(info.device_nbr27(), oracle.neighbours(L)), f"nbr27 level {l}"
    F, s = d["ratios"][0], d["ratios"][0]
    Li, Lo = d["olv"][0], d["olv"][1]
    field = torch.empty((Lo.Ntot, F ** 3), dtype=torch.int32, device="cuda")
    hch.hch_field_build(dlv, 0, F, s, 0, field, None)
    assert np.array_equal(field.cpu().numpy(), oracle.field_indices(Li, Lo, F, s, 0))


def _fields(case, level_in, F, stride, pad, Li, Lo):
    field = torch.full((Lo.Ntot, F ** 3), -7, dtype=torch.int32, device="cuda")
    field_t = torch.full((Li.Ntot, F ** 3), -7, dtype=torch.int32, device="cuda")
    hch.hch_field_build(case["glv"], level_in, F, stride, pad, field, field_t)
    return field, field_t


def _cases(d):
    r0 = d["ratios"][0]
    out = [(0, r0, r0, 0, 0, 1), (0, r0 + 2, r0, 1, 0, 1)]        # (level_in, F, stride, pad, li, lo)
    if len(d["ratios"]) > 1:
        out.append((0, 6, r0 * d["ratios"][1], 0, 0, 2))           # across both ratios: stride 6
        out.append((1, 2, 2, 0, 1, 2))
    return out


def test_ratio_field_lists_bit_exact(oracle, ratio_case):
    d = ratio_case
    for level_in, F, stride, pad, li, lo in _cases(d):
        Li, Lo = d["olv"][li], d["olv"][lo]
        field, field_t = _fields(d, level_in, F, stride, pad, Li, Lo)
        want = oracle.field_indices(Li, Lo, F, stride, pad)
        assert np.array_equal(field.cpu().numpy(), want), (F, stride, pad)
        want_t = np.full((Li.Ntot, F ** 3), -1, np.int32)
        o, row = np.nonzero(want >= 0)
        want_t[want[o, row], row] = o
        assert np.array_equal(field_t.cpu().numpy(), want_t), (F, stride, pad)


def test_ratio_conv_and_pooling(oracle, ratio_case):
    """Strided convolution (forward, both gradients), max pooling with switches and average
    pooling between levels in ratio 3 / 5 / 6."""
    d = ratio_case
    F32 = hch.HCH_F32
    for level_in, F, stride, pad, li, lo in _cases(d):
        Li, Lo = d["olv"][li], d["olv"][lo]
        F3 = F ** 3
        field, field_t = _fields(d, level_in, F, stride, pad, Li, Lo)
        c_in, c_out = 8, 16
        X = S.gaussian((Li.Ntot, c_in), 1.0, 151)
        W = S.gaussian((F3, c_in, c_out), 0.1, 152)
        G = S.gaussian((Lo.Ntot, c_out), 1.0, 153)
        Xp, Wp, Gp = oracle.to_paper_X(X), oracle.to_paper_W(W), oracle.to_paper_X(G)
        ws = workspace(max(hch.hch_sconv_workspace_bytes(d["glv"], level_in, F, stride, c_in, c_out, F32, k)
                           for k in (hch.HCH_WS_FWD, hch.HCH_WS_BWD_DATA, hch.HCH_WS_BWD_WEIGHT)))
        Y = torch.full((Lo.Ntot, c_out), float("nan"), dtype=torch.float32, device="cuda")
        hch.hch_sconv_fwd(d["glv"], level_in, F, stride, F32, dev(X), dev(W), Y, field, c_in, c_out, ws)
        assert_close(Y.cpu().numpy(), oracle.sconv_fwd(Li, Lo, Xp, Wp, F, stride, pad).T, what=f"fwd {F},{stride}")
        dW = torch.full((F3, c_in, c_out), float("nan"), dtype=torch.float32, device="cuda")
        hch.hch_sconv_bwd_weight(d["glv"], level_in, F, stride, F32, dev(X), dev(G), dW, field, c_in, c_out, ws)
        want_dW = oracle.sconv_bwd_weight(Li, Lo, Xp, Gp, F, stride, pad).reshape(c_out, c_in, F3).transpose(2, 1, 0)
        assert_close(dW.cpu().numpy(), want_dW, what=f"dW {F},{stride}")
        dX = torch.full((Li.Ntot, c_in), float("nan"), dtype=torch.float32, device="cuda")
        hch.hch_sconv_bwd_data(d["glv"], level_in, F, stride, F32, dev(G), dev(W), dX, field_t, c_in, c_out, ws)
        assert_close(dX.cpu().numpy(), oracle.sconv_bwd_data(Li, Lo, Gp, Wp, c_in, F, stride, pad).T, what=f"dX {F},{stride}")

        for c in (8, 5):
            Xc = S.gaussian((Li.Ntot, c), 1.0, 161)
            Gc = S.gaussian((Lo.Ntot, c), 1.0, 162)
            # average pooling: weights 1/F^3, empty entries count as zero
            A = torch.full((Lo.Ntot, c), float("nan"), dtype=torch.float32, device="cuda")
            hch.hch_spool_avg_fwd(d["glv"], level_in, F, stride, dev(Xc), field, A, c)
            assert_close(A.cpu().numpy(), oracle.avgpool_fwd(Li, Lo, oracle.to_paper_X(Xc), F, stride, pad).T, what="avg fwd")
            dA = torch.full((Li.Ntot, c), float("nan"), dtype=torch.float32, device="cuda")
            hch.hch_spool_avg_bwd(d["glv"], level_in, F, stride, pad, dev(Gc), None, field_t, dA, c)
            assert_close(dA.cpu().numpy(), oracle.avgpool_bwd(Li, Lo, oracle.to_paper_X(Gc), F, stride, pad).T, what="avg bwd")
            if F == stride and pad == 0:   # the fields partition the input level: the form that writes through `field`
                dA2 = torch.full((Li.Ntot, c), float("nan"), dtype=torch.float32, device="cuda")
                hch.hch_spool_avg_bwd(d["glv"], level_in, F, stride, pad, dev(Gc), field, None, dA2, c)
                assert torch.equal(dA, dA2)
            if F > stride:
                continue        # overlapping fields: the oracle's switch routing is defined for disjoint ones
            P = torch.full((Lo.Ntot, c), float("nan"), dtype=torch.float32, device="cuda")
            sw = torch.full((Lo.Ntot, c), -9, dtype=torch.int32, device="cuda")
            hch.hch_spool_max_fwd(d["glv"], level_in, F, stride, dev(Xc), field, P, sw, c)
            Po, swo = oracle.pool_max_fwd(Li, Lo, oracle.to_paper_X(Xc), F, stride, pad)
            assert np.array_equal(sw.cpu().numpy(), swo.T)
            assert np.array_equal(P.cpu().numpy(), Po.T.astype(np.float32))
            dP = torch.full((Li.Ntot, c), float("nan"), dtype=torch.float32, device="cuda")
            hch.hch_spool_max_bwd(d["glv"], level_in, F, stride, pad, dev(Gc), sw, None, field_t, dP, c)
            want = oracle.pool_max_bwd(Li.Ntot, oracle.to_paper_X(Gc), swo).T
            assert np.array_equal(dP.cpu().numpy(), want.astype(np.float32))
            if F == stride and pad == 0:
                dP2 = torch.full((Li.Ntot, c), float("nan"), dtype=torch.float32, device="cuda")
                hch.hch_spool_max_bwd(d["glv"], level_in, F, stride, pad, dev(Gc), sw, field, None, dP2, c)
                assert torch.equal(dP, dP2)


def test_field_pooling_equals_child_pooling(oracle):
    """On levels in ratio 2, pooling through the 2^3 field rows gives the bits of hch_pool_* and
    hch_avgpool_*."""
    coords, offs, _ = S.config_batch(2, batch=3, u=64)
    glv = hch.hch_build_levels(coords, offs, 64, 2)
    nf, nc = glv.n(0), glv.n(1)
    field = torch.empty((nc, 8), dtype=torch.int32, device="cuda")
    field_t = torch.empty((nf, 8), dtype=torch.int32, device="cuda")
    hch.hch_field_build(glv, 0, 2, 2, 0, field, field_t)
    for c in (16, 7):
        X, G = dev(S.gaussian((nf, c), 1.0, 171)), dev(S.gaussian((nc, c), 1.0, 172))
        P1, P2 = (torch.empty((nc, c), dtype=torch.float32, device="cuda") for _ in range(2))
        s1, s2 = (torch.empty((nc, c), dtype=torch.int32, device="cuda") for _ in range(2))
        hch.hch_pool_fwd(glv, 0, X, P1, s1, c)
        hch.hch_spool_max_fwd(glv, 0, 2, 2, X, field, P2, s2, c)
        assert torch.equal(P1, P2) and torch.equal(s1, s2)
        d1, d2 = (torch.empty((nf, c), dtype=torch.float32, device="cuda") for _ in range(2))
        hch.hch_pool_bwd(glv, 0, G, s1, d1, c)
        hch.hch_spool_max_bwd(glv, 0, 2, 2, 0, G, s2, None, field_t, d2, c)
        assert torch.equal(d1, d2)
        d2.fill_(float("nan"))
        hch.hch_spool_max_bwd(glv, 0, 2, 2, 0, G, s2, field, None, d2, c)
        assert torch.equal(d1, d2)
        hch.hch_avgpool_fwd(glv, 0, X, P1, c)
        hch.hch_spool_avg_fwd(glv, 0, 2, 2, X, field, P2, c)
        assert torch.equal(P1, P2)
        hch.hch_avgpool_bwd(glv, 0, G, d1, c)
        hch.hch_spool_avg_bwd(glv, 0, 2, 2, 0, G, None, field_t, d2, c)
        assert torch.equal(d1, d2)
        d2.fill_(float("nan"))
        hch.hch_spool_avg_bwd(glv, 0, 2, 2, 0, G, field, None, d2, c)
        assert torch.equal(d1, d2)


def test_padded_partition_pooling_backward(oracle):
    """F = stride with padding: the fields still tile the grid, but an input voxel can lie in the
    field of a position that is unoccupied on the output level, where no forward row reaches it.
    Its gradient is zero; dX is prefilled with NaN to show that every row is written.  With
    padding the backward calls must go through field_t, whether or not `field` is passed."""
    coords, offs, _ = S.config_batch(2, batch=3, u=64)
    olv = oracle.build_hierarchy(coords, offs, 64, 2)
    glv = hch.hch_build_levels(coords, offs, 64, 2)
    Li, Lo = olv[0], olv[1]
    F, stride, pad = 2, 2, 1
    field = torch.empty((Lo.Ntot, 8), dtype=torch.int32, device="cuda")
    field_t = torch.empty((Li.Ntot, 8), dtype=torch.int32, device="cuda")
    hch.hch_field_build(glv, 0, F, stride, pad, field, field_t)
    want_field = oracle.field_indices(Li, Lo, F, stride, pad)
    assert np.array_equal(field.cpu().numpy(), want_field)
    covered = np.zeros(Li.Ntot, bool)
    covered[want_field[want_field >= 0]] = True
    assert not covered.all(), "the case must contain input voxels that no occupied output's field holds"
    for c in (8, 5):
        Xc, Gc = S.gaussian((Li.Ntot, c), 1.0, 181), S.gaussian((Lo.Ntot, c), 1.0, 182)
        want_avg = oracle.avgpool_bwd(Li, Lo, oracle.to_paper_X(Gc), F, stride, pad).T
        assert np.all(want_avg[~covered] == 0)
        for f in (field, None):
            dA = torch.full((Li.Ntot, c), float("nan"), dtype=torch.float32, device="cuda")
            hch.hch_spool_avg_bwd(glv, 0, F, stride, pad, dev(Gc), f, field_t, dA, c)
            assert_close(dA.cpu().numpy(), want_avg, what="avg bwd, padded partition")
        P = torch.full((Lo.Ntot, c), float("nan"), dtype=torch.float32, device="cuda")
        sw = torch.full((Lo.Ntot, c), -9, dtype=torch.int32, device="cuda")
        hch.hch_spool_max_fwd(glv, 0, F, stride, dev(Xc), field, P, sw, c)
        Po, swo = oracle.pool_max_fwd(Li, Lo, oracle.to_paper_X(Xc), F, stride, pad)
        assert np.array_equal(sw.cpu().numpy(), swo.T) and np.array_equal(P.cpu().numpy(), Po.T.astype(np.float32))
        # an output voxel whose padded field is empty has the switch -1 and routes nothing
        want_max = oracle.pool_max_bwd(Li.Ntot, oracle.to_paper_X(Gc), swo)
        for f in (field, None):
            dP = torch.full((Li.Ntot, c), float("nan"), dtype=torch.float32, device="cuda")
            hch.hch_spool_max_bwd(glv, 0, F, stride, pad, dev(Gc), sw, f, field_t, dP, c)
            assert np.array_equal(dP.cpu().numpy(), want_max.T.astype(np.float32))
        with pytest.raises(hch.HchError) as ei:        # the forward rows alone cannot serve a padded field
            hch.hch_spool_max_bwd(glv, 0, F, stride, pad, dev(Gc), sw, field, None, dP, c)
        assert ei.value.status == 1
        with pytest.raises(hch.HchError) as ei:
            hch.hch_spool_avg_bwd(glv, 0, F, stride, pad, dev(Gc), field, None, dA, c)
        assert ei.value.status == 1


def test_ratio_errors(oracle, ratio_case):
    d = ratio_case
    glv = d["glv"]
    n0, n1 = glv.n(0), glv.n(1)
    X = torch.zeros((n0, 4), dtype=torch.float32, device="cuda")
    Y = torch.zeros((n1, 4), dtype=torch.float32, device="cuda")
    sw = torch.zeros((n1, 4), dtype=torch.int32, device="cuda")
    with pytest.raises(hch.HchError) as ei:            # no child lists between levels in ratio 3 / 5
        hch.hch_pool_fwd(glv, 0, X, Y, sw, 4)
    assert ei.value.status == 5
    with pytest.raises(hch.HchError) as ei:
        hch.hch_avgpool_fwd(glv, 0, X, Y, 4)
    assert ei.value.status == 5
    f = torch.empty((n1, 27), dtype=torch.int32, device="cuda")
    with pytest.raises(hch.HchError) as ei:            # no level 2 or 4 times coarser than level 0
        hch.hch_field_build(glv, 0, 3, 2 if d["ratios"][0] != 2 else 4, 1, f, None)
    assert ei.value.status == 1
    for bad in ([1], [0], [-3]):
        with pytest.raises(hch.HchError) as ei:
            hch.hch_build_levels_ratios(d["coords"], d["offs"], d["u"], bad)
        assert ei.value.status == 1
    with pytest.raises(hch.HchError):                   # a level of side 1 cannot be coarsened further
        hch.hch_build_levels_ratios(d["coords"], d["offs"], d["u"], [d["u"], 2])
