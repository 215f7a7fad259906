"""The entry point that allocates nothing (caat_norm_bwd_static: partial sums in a fixed device array inside the
library instead of a caller's workspace) against the entry point it is a variant of (caat_norm_bwd), through the C ABI:
two calls in a row, the second on a smaller input, so that what the first call left in the shared array must not leak
into the second."""
import numpy as np
import pytest

from oracle import caat_oracle as O
from paper_2506_19645_amd import binding as B
from paper_2506_19645_amd import inputs as I
from tests.util import assert_close, bits_to_f64

pytestmark = pytest.mark.gpu


def _run(static, d, layernorm, T, n, h, hs, scale):
    import torch
    kind = B.LAYERNORM if layernorm else B.RMSNORM
    x, gam = B.to_device(d["R"]), B.to_device(d["gamma"])
    bet = B.to_device(d["beta"]) if layernorm else None
    y = torch.empty_like(x)
    mean = torch.empty(T * n, dtype=torch.float32, device="cuda") if layernorm else None
    rstd = torch.empty(T * n, dtype=torch.float32, device="cuda")
    B.norm_fwd(x, gam, bet, y, mean, rstd, kind, T, n, h, 1e-5)
    dy, dres = B.to_device(d["dXo"]), B.to_device(d["dRo"])
    g_out, g_sc = torch.full_like(x, float("nan")), torch.full_like(x, float("nan"))
    dgamma = torch.full((h,), float("nan"), dtype=torch.float32, device="cuda")
    dbeta = torch.full((h,), float("nan"), dtype=torch.float32, device="cuda") if layernorm else None
    if static:
        B.norm_bwd_static(dy, dres, x, gam, mean, rstd, g_out, g_sc, dgamma, dbeta, kind, T, n, h, hs, scale)
    else:
        ws = torch.empty(B.norm_bwd_workspace_bytes(T, n, h), dtype=torch.uint8, device="cuda")
        B.norm_bwd(dy, dres, x, gam, mean, rstd, g_out, g_sc, dgamma, dbeta, kind, T, n, h, hs, scale, ws)
    torch.cuda.synchronize()
    return {"g": B.to_host_bits(g_out), "gs": B.to_host_bits(g_sc), "dgamma": dgamma.cpu().numpy(),
            "dbeta": dbeta.cpu().numpy() if layernorm else None}


@pytest.mark.parametrize("layernorm", [True, False])
@pytest.mark.parametrize("big,small", [((4, 1500, 2048), (2, 77, 520)),      # wave-per-row kernel, 512 then 39 partial rows
                                       ((2, 1000, 8192), (1, 30, 4104))])    # workgroup-per-row kernel (h > 4096)
def test_norm_bwd_static_matches_norm_bwd_on_two_calls_in_a_row(layernorm, big, small):
    for k, (T, n, h) in enumerate((big, small)):
        d = I.make_norm_inputs(T, n, h, layernorm, seed=90 + k)
        hs, scale = (h // 2 + 3, 1.5) if k == 0 else (h // 4 // 8 * 8, 1.0)
        want = _run(False, d, layernorm, T, n, h, hs, scale)
        got = _run(True, d, layernorm, T, n, h, hs, scale)
        # same kernels, same launch shape, same summation order: the bf16 outputs carry the same bits
        assert np.array_equal(got["g"], want["g"]) and np.array_equal(got["gs"], want["gs"]), (k, T, n, h)
        np.testing.assert_allclose(got["dgamma"], want["dgamma"], rtol=1e-6, atol=1e-6)
        if layernorm:
            np.testing.assert_allclose(got["dbeta"], want["dbeta"], rtol=1e-6, atol=1e-6)
        # and both are the oracle's gradients
        w = {key: O.widen_bf16(v) for key, v in d.items()}
        dn, dgm, dbm = O.norm_bwd(w["dXo"], w["R"], w["gamma"], O.LAYERNORM if layernorm else O.RMSNORM, 1e-5)
        assert_close(bits_to_f64(got["g"]), w["dRo"] + dn, "g")
        assert_close(got["dgamma"], dgm.sum(0), "dgamma", tol=5e-3)
        if layernorm:
            assert_close(got["dbeta"], dbm.sum(0), "dbeta", tol=5e-3)


def test_norm_bwd_static_refuses_what_its_scratch_cannot_hold():
    import torch
    T, n, h = 1, 2056, 8192                       # 257 partial rows of 8 h bytes: 8 KiB more than the 16 MiB array
    x = torch.zeros(T * n * h, dtype=torch.bfloat16, device="cuda")
    g = torch.full_like(x, 7.0)
    rstd = torch.ones(T * n, dtype=torch.float32, device="cuda")
    dgamma = torch.full((h,), 7.0, dtype=torch.float32, device="cuda")
    st = B.norm_bwd_static(x, None, x, x, None, rstd, g, None, dgamma, None, B.RMSNORM, T, n, h, 0, 1.0, check=False)
    torch.cuda.synchronize()
    assert st == B.ESCRATCH
    assert bool((g == 7.0).all()) and bool((dgamma == 7.0).all())      # nothing was launched
