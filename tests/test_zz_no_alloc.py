"""hch_conv_bwd_weight_noalloc: the weight gradient for callers that cannot allocate (partial sums
in the library's built-in scratch array) against hch_conv_bwd_weight with a caller's workspace,
which the parity tests check against the oracle.  Same kernels and same split plan, so the results
must agree bit for bit; two calls in a row, the second on a smaller input, so that what the
first call left in the array would show.  Collected last: it must pass alone in a fresh process
and after everything else."""
import numpy as np
import pytest

import synth_shapes as S

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
hch = pytest.importorskip("paper_1803_11385_amd")


def _workspace(nbytes):
    t = torch.empty(int(nbytes) + 256, dtype=torch.uint8, device="cuda")
    off = (-t.data_ptr()) % 256
    return t[off: off + int(nbytes)]


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda")


def _both(glv, level, dtype, X, G, c_in, c_out):
    need = hch.hch_conv_workspace_bytes(glv, level, c_in, c_out, dtype, hch.HCH_WS_BWD_WEIGHT, hch.HCH_ALGO_FUSED)
    assert need <= hch.HCH_NOALLOC_SCRATCH_BYTES
    want = torch.full((27, c_in, c_out), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_conv_bwd_weight(glv, level, dtype, X, G, want, c_in, c_out, _workspace(need), hch.HCH_ALGO_FUSED)
    got = torch.full((27, c_in, c_out), float("nan"), dtype=torch.float32, device="cuda")
    hch.hch_conv_bwd_weight_noalloc(glv, level, dtype, X, G, got, c_in, c_out)
    torch.cuda.synchronize()
    return got, want


def test_noalloc_weight_gradient_two_calls_in_a_row(oracle):
    coords, offs, _ = S.config_batch(3, batch=4, u=64)
    glv = hch.hch_build_levels(coords, offs, 64, 3)
    olv = oracle.build_hierarchy(coords, offs, 64, 3)
    # first call: the finest level, 32 -> 64 (a split reduction over many slices); second call: a
    # coarser level with fewer channels, i.e. fewer and smaller partial sums in the same array;
    # third: bf16 inputs on the bf16 matrix instruction
    for level, c_in, c_out, dtype in ((0, 32, 64, hch.HCH_F32), (2, 5, 7, hch.HCH_F32), (1, 16, 32, hch.HCH_BF16),
                                      (0, 32, 64, hch.HCH_F32)):
        n = glv.n(level)
        X, G = S.gaussian((n, c_in), 1.0, 901 + level), S.gaussian((n, c_out), 1.0, 911 + level)
        if dtype == hch.HCH_BF16:
            X, G = S.to_bf16_grid(X), S.to_bf16_grid(G)
            Xd, Gd = _dev(S.bf16_bits(X).view(np.int16)), _dev(S.bf16_bits(G).view(np.int16))
        else:
            Xd, Gd = _dev(X), _dev(G)
        got, want = _both(glv, level, dtype, Xd, Gd, c_in, c_out)
        assert torch.equal(got, want), (level, c_in, c_out)
        # and against the oracle (Eq.7), to the bar of the other parity tests
        ref = oracle.from_paper_W(oracle.conv_bwd_weight(olv[level], oracle.to_paper_X(X), oracle.to_paper_X(G)), c_in)
        g = got.cpu().numpy().astype(np.float64)
        rms = float(np.sqrt((ref ** 2).mean()))
        assert np.all(np.abs(g - ref) <= 1e-4 * (np.abs(ref) + rms))


def test_noalloc_limits_and_errors():
    """The partial sums of every product the split planning produces fit the built-in array (the
    planning fills one round of workgroups, which bounds them by 24 MiB whatever the level and the
    channel counts, so the HCH_EWORKSPACE guard only fires if the planning changes); bad arguments
    are refused before anything is launched."""
    coords, offs, _ = S.config_batch(3, batch=4, u=64)
    glv = hch.hch_build_levels(coords, offs, 64, 3)
    worst = 0
    for level in range(3):
        for dtype in (hch.HCH_F32, hch.HCH_BF16):
            for c_in in (1, 3, 4, 16, 24, 64, 100, 128, 256, 512):
                for c_out in (1, 4, 16, 32, 64, 96, 128, 256, 512):
                    worst = max(worst, hch.hch_conv_workspace_bytes(glv, level, c_in, c_out, dtype,
                                                                    hch.HCH_WS_BWD_WEIGHT, hch.HCH_ALGO_FUSED))
    assert 0 < worst <= hch.HCH_NOALLOC_SCRATCH_BYTES, worst
    n = glv.n(0)
    X = torch.zeros((n, 8), dtype=torch.float32, device="cuda")
    G = torch.zeros((n, 8), dtype=torch.float32, device="cuda")
    dW = torch.full((27, 8, 8), 7.0, dtype=torch.float32, device="cuda")
    lib = hch.load_library()
    import ctypes as C
    vp = C.c_void_p
    h, s = glv.handle, vp(torch.cuda.current_stream().cuda_stream)
    x, g, w = vp(X.data_ptr()), vp(G.data_ptr()), vp(dW.data_ptr())
    assert lib.hch_conv_bwd_weight_noalloc(h, 3, 0, x, g, w, 8, 8, s) == 1        # no such level
    assert lib.hch_conv_bwd_weight_noalloc(h, 0, 7, x, g, w, 8, 8, s) == 1        # unknown dtype
    assert lib.hch_conv_bwd_weight_noalloc(h, 0, 0, vp(None), g, w, 8, 8, s) == 1  # null input
    assert lib.hch_conv_bwd_weight_noalloc(h, 0, 0, x, g, w, 0, 8, s) == 1        # channel count
    assert lib.hch_conv_bwd_weight_noalloc(None, 0, 0, x, g, w, 8, 8, s) == 1     # no level set
    torch.cuda.synchronize()
    assert bool((dW == 7.0).all()), "nothing may be written on error"
