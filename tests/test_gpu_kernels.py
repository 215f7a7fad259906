"""GPU parity of the individual HIP kernels against the CPU oracle, called through the C ABI.
Bit-exact for channel selection / indexing, <= 2e-2 relative for floating point (bf16 storage, fp32 accumulate)."""
import numpy as np
import pytest

from oracle import caat_oracle as O
from paper_2506_19645_amd import binding as B
from paper_2506_19645_amd import inputs as I
from tests.util import assert_close, bits_to_f64, f64_to_bits, ulp_distance_bf16

pytestmark = pytest.mark.gpu


def _torch():
    import torch
    return torch


# ------------------------------------------------------------------------------------------ partial sync
@pytest.mark.parametrize("T", [1, 2, 3, 4, 8, 16])
def test_partial_sync_integer_bit_exact(T):
    """Small-integer inputs make every sum exact: GPU bits must equal the oracle's, for every hs edge case."""
    torch = _torch()
    n, h = 37, 40
    d = I.make_sync_inputs(T, n, h, seed=10 + T, integer=True)
    Zt, R = O.widen_bf16(d["Zt"]), O.widen_bf16(d["R"])
    y, r = B.to_device(d["Zt"]), B.to_device(d["R"])
    for hs in (0, 1, 7, 8, 9, 16, h - 1, h):
        for scale in (1.0, 2.0):
            for use_res in (False, True):
                want = O.partial_channel_reduce(Zt, hs, scale) + (R if use_res else 0.0)
                out = torch.full_like(y, float("nan"))
                B.partial_sync(y, r if use_res else None, out, T, n, h, hs, scale)
                torch.cuda.synchronize()
                got = B.to_host_bits(out)
                assert np.array_equal(got, f64_to_bits(want)), (T, hs, scale, use_res)
                # in place
                y2 = y.clone()
                B.partial_sync(y2, r if use_res else None, y2, T, n, h, hs, scale)
                torch.cuda.synchronize()
                assert np.array_equal(B.to_host_bits(y2), got), ("inplace", T, hs, scale, use_res)


@pytest.mark.parametrize("T,n,h,hs", [(2, 256, 768, 384), (4, 333, 2048, 1000), (8, 129, 4096, 2048), (5, 64, 264, 131),
                                        (16, 70, 8192, 4096)])
def test_partial_sync_random_values(T, n, h, hs):
    torch = _torch()
    d = I.make_sync_inputs(T, n, h, seed=3)
    Zt, R = O.widen_bf16(d["Zt"]), O.widen_bf16(d["R"])
    y, r = B.to_device(d["Zt"]), B.to_device(d["R"])
    # in place, no residual: only shared channels may change, and they are identical on all ranks
    y2 = y.clone()
    B.partial_sync(y2, None, y2, T, n, h, hs, 1.0)
    torch.cuda.synchronize()
    got = B.to_host_bits(y2)
    assert np.array_equal(got[:, :, hs:], d["Zt"][:, :, hs:])                 # private channels: bits untouched
    for m in range(1, T):
        assert np.array_equal(got[m, :, :hs], got[0, :, :hs])                  # shared: same bits on every rank
    want = O.partial_channel_reduce(Zt, hs)
    # fp32 ascending-order sum then one rounding: within 1 bf16 ulp of the exactly rounded fp64 sum
    assert ulp_distance_bf16(got, f64_to_bits(want)).max() <= 1
    assert_close(bits_to_f64(got), want, "pcr")
    # with residual, out of place
    out = torch.empty_like(y)
    B.partial_sync(y, r, out, T, n, h, hs, 1.0)
    torch.cuda.synchronize()
    assert_close(bits_to_f64(B.to_host_bits(out)), want + R, "pcr+res")
    assert np.array_equal(B.to_host_bits(y), d["Zt"])                           # input not modified


def test_partial_sync_p0_p1():
    torch = _torch()
    T, n, h = 4, 100, 512
    d = I.make_sync_inputs(T, n, h, seed=4)
    y = B.to_device(d["Zt"])
    y0 = y.clone()
    B.partial_sync(y0, None, y0, T, n, h, 0, 1.0)            # p = 0: nothing is summed, bits unchanged
    torch.cuda.synchronize()
    assert np.array_equal(B.to_host_bits(y0), d["Zt"])
    y1 = y.clone()
    B.partial_sync(y1, None, y1, T, n, h, h, 1.0)            # p = 1: plain all-reduce
    torch.cuda.synchronize()
    got = bits_to_f64(B.to_host_bits(y1))
    want = O.widen_bf16(d["Zt"]).sum(axis=0)
    for m in range(T):
        assert_close(got[m], want, "allreduce")
        assert np.array_equal(got[m], got[0])


def test_partial_sync_empty():
    torch = _torch()
    y = torch.zeros(8, dtype=torch.bfloat16, device="cuda")
    assert B.partial_sync(y, None, y, 2, 0, 8, 8) == B.OK
    torch.cuda.synchronize()


# ------------------------------------------------------------------------------------------ fused reduce + norm
@pytest.mark.parametrize("layernorm", [False, True])
@pytest.mark.parametrize("T,n,h,hs", [(2, 37, 40, 8), (4, 9, 2048, 1024), (8, 5, 4096, 2048), (8, 3, 8192, 4096),
                                        (16, 6, 4096, 2048), (16, 4, 264, 264), (4, 3, 520, 512)])
def test_partial_sync_norm_fwd_integer_bit_exact(layernorm, T, n, h, hs):
    """The one-launch reduce + residual + norm: with small-integer partial sums and residuals every sum is exact, so
    the shared channels of R' must carry exactly the oracle's bits on every rank and the private channels must keep
    theirs; the normalised copy is compared with the oracle's norm of that R'."""
    torch = _torch()
    kind = O.LAYERNORM if layernorm else O.RMSNORM
    d = I.make_sync_inputs(T, n, h, seed=70 + T, integer=True)
    dn = I.make_norm_inputs(T, n, h, layernorm, seed=71 + T)
    io_bits = d["Zt"].copy()
    io_bits[:, :, hs:] = dn["R"][:, :, hs:]                   # private channels: already final, arbitrary values
    Zt, R = O.widen_bf16(d["Zt"]), O.widen_bf16(d["R"])
    want_rp = O.widen_bf16(io_bits)
    want_rp[:, :, :hs] = O.partial_channel_reduce(Zt, hs)[:, :, :hs] + R[:, :, :hs]
    gam, bet = O.widen_bf16(dn["gamma"]), (O.widen_bf16(dn["beta"]) if layernorm else None)
    want_x, _, want_rstd = O.norm_fwd(want_rp, gam, bet, kind, 1e-5)
    io, res = B.to_device(io_bits), B.to_device(d["R"])
    x_out = torch.full_like(io, float("nan"))
    mean = torch.empty(T * n, dtype=torch.float32, device="cuda") if layernorm else None
    rstd = torch.empty(T * n, dtype=torch.float32, device="cuda")
    B.partial_sync_norm_fwd(io, res, B.to_device(dn["gamma"]), B.to_device(dn["beta"]) if layernorm else None, x_out,
                            mean, rstd, kind, T, n, h, hs, 1e-5)
    torch.cuda.synchronize()
    got = B.to_host_bits(io)
    assert np.array_equal(got[:, :, :hs], f64_to_bits(want_rp[:, :, :hs]))      # exact sums + residual, every rank
    assert np.array_equal(got[:, :, hs:], io_bits[:, :, hs:])                   # private channels: bits untouched
    assert_close(bits_to_f64(B.to_host_bits(x_out)), want_x, "fused norm output")
    assert_close(rstd.cpu().numpy().reshape(T, n, 1), want_rstd, "rstd", tol=1e-4)
    if layernorm:
        assert_close(mean.cpu().numpy().reshape(T, n), want_rp.mean(-1), "mean", tol=1e-4)


def test_partial_sync_norm_fwd_shapes_not_taken():
    torch = _torch()
    buf = torch.zeros(16 * 2 * 8192, dtype=torch.bfloat16, device="cuda")
    rstd = torch.zeros(64, dtype=torch.float32, device="cuda")
    call = lambda T, n, h, hs: B.partial_sync_norm_fwd(buf, buf, buf, None, buf, None, rstd, B.RMSNORM, T, n, h, hs, 1e-5,
                                                       check=False)
    assert call(2, 2, 64, 12) == B.EUNSUPPORTED       # a 16-byte group straddles hs
    assert call(2, 2, 64, 0) == B.EUNSUPPORTED        # nothing shared
    assert call(3, 2, 64, 32) == B.EUNSUPPORTED       # rank counts without an instantiation
    assert call(16, 2, 8192, 4096) == B.EUNSUPPORTED  # T = 16 is taken up to h = 4096
    assert call(2, 2, 64, 72) == B.ESHAPE
    assert call(2, 0, 64, 32) == B.OK
    torch.cuda.synchronize()


# ------------------------------------------------------------------------------------------ norms
@pytest.mark.parametrize("layernorm", [True, False])
@pytest.mark.parametrize("T,n,h", [(2, 33, 64), (2, 256, 768), (3, 70, 520), (4, 65, 2048), (2, 40, 4096), (1, 9, 8192)])
def test_norm_fwd_bwd(layernorm, T, n, h):
    torch = _torch()
    kind = O.LAYERNORM if layernorm else O.RMSNORM
    d = I.make_norm_inputs(T, n, h, layernorm, seed=h + T)
    w = {k: O.widen_bf16(v) for k, v in d.items()}
    eps = 1e-5
    want_y, _, want_rstd = O.norm_fwd(w["R"], w["gamma"], w.get("beta"), kind, eps)
    x, gam = B.to_device(d["R"]), B.to_device(d["gamma"])
    bet = B.to_device(d["beta"]) if layernorm else None
    y = torch.empty_like(x)
    mean = torch.empty(T * n, dtype=torch.float32, device="cuda") if layernorm else None
    rstd = torch.empty(T * n, dtype=torch.float32, device="cuda")
    B.norm_fwd(x, gam, bet, y, mean, rstd, kind, T, n, h, eps)
    torch.cuda.synchronize()
    assert_close(bits_to_f64(B.to_host_bits(y)), want_y, "norm_fwd")
    assert_close(rstd.cpu().numpy().reshape(T, n, 1), want_rstd, "rstd", tol=1e-4)
    if layernorm:
        assert_close(mean.cpu().numpy().reshape(T, n), w["R"].mean(-1), "mean", tol=1e-4)
    # backward, with the private-scaled copy
    hs, scale = (h // 2 + 3), 1.5
    dn, dgm, dbm = O.norm_bwd(w["dXo"], w["R"], w["gamma"], kind, eps)
    want_g = w["dRo"] + dn
    want_gs = want_g.copy()
    want_gs[:, :, hs:] *= scale
    dy, dres = B.to_device(d["dXo"]), B.to_device(d["dRo"])
    g_out, g_sc = torch.empty_like(x), torch.empty_like(x)
    dgamma = torch.empty(h, dtype=torch.float32, device="cuda")
    dbeta = torch.empty(h, dtype=torch.float32, device="cuda") if layernorm else None
    ws = torch.empty(B.norm_bwd_workspace_bytes(T, n, h), dtype=torch.uint8, device="cuda")
    B.norm_bwd(dy, dres, x, gam, mean, rstd, g_out, g_sc, dgamma, dbeta, kind, T, n, h, hs, scale, ws)
    torch.cuda.synchronize()
    assert_close(bits_to_f64(B.to_host_bits(g_out)), want_g, "norm_bwd g")
    assert_close(bits_to_f64(B.to_host_bits(g_sc)), want_gs, "norm_bwd g_scaled")
    assert_close(dgamma.cpu().numpy(), dgm.sum(0), "dgamma", tol=5e-3)
    if layernorm:
        assert_close(dbeta.cpu().numpy(), dbm.sum(0), "dbeta", tol=5e-3)
    # no residual gradient, no scaled copy
    g2 = torch.empty_like(x)
    B.norm_bwd(dy, None, x, gam, mean, rstd, g2, None, dgamma, dbeta, kind, T, n, h, 0, 1.0, ws)
    torch.cuda.synchronize()
    assert_close(bits_to_f64(B.to_host_bits(g2)), dn, "norm_bwd no-res")


# ------------------------------------------------------------------------------------------ shard GEMM
GEMM_SHAPES = [(1, 32, 32, 16), (2, 256, 256, 64), (3, 300, 264, 200), (2, 513, 520, 1376), (1, 1000, 776, 72),
               (2, 8, 8, 8)]


@pytest.mark.parametrize("G,M,N,K", GEMM_SHAPES)
@pytest.mark.parametrize("layout", [B.GEMM_NT, B.GEMM_NN, B.GEMM_TN])
def test_gemm_layouts(layout, G, M, N, K):
    torch = _torch()
    if layout == B.GEMM_TN and M % 8:
        M = (M + 7) // 8 * 8
    d = I.make_gemm_inputs(G, M, N, K, seed=M + N + K, std_a=1.0, std_b=0.05)
    a, b = O.widen_bf16(d["a"]), O.widen_bf16(d["b"])          # a [G,M,K], b [G,N,K]
    want = np.einsum("gmk,gnk->gmn", a, b)
    if layout == B.GEMM_NT:
        da, db, lda, ldb = d["a"], d["b"], K, K
    elif layout == B.GEMM_NN:
        da, db, lda, ldb = d["a"], np.ascontiguousarray(d["b"].transpose(0, 2, 1)), K, N
    else:
        da = np.ascontiguousarray(d["a"].transpose(0, 2, 1))
        db = np.ascontiguousarray(d["b"].transpose(0, 2, 1))
        lda, ldb = M, N
    ta, tb = B.to_device(da), B.to_device(db)
    c = torch.full((G, M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    B.gemm_bf16(ta, tb, c, layout, G, M, N, K, lda, ldb, N, M * K, N * K, M * N)
    torch.cuda.synchronize()
    assert_close(bits_to_f64(B.to_host_bits(c)), want, "gemm layout %d" % layout, tol=5e-3)


def _random_gemm_shapes(count, seed):
    r = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        G = int(r.integers(1, 4))
        M = int(r.choice([8, 40, 64, 72, 200, 256, 264, 520, 776]))
        N = int(r.choice([8, 32, 64, 136, 256, 264, 512, 600]))
        K = int(r.choice([8, 24, 56, 64, 72, 128, 136, 200, 328, 1032]))
        out.append((int(r.integers(0, 3)), G, M, N, K))
    return out


@pytest.mark.parametrize("layout,G,M,N,K", _random_gemm_shapes(36, seed=2024))
def test_gemm_random_shapes(layout, G, M, N, K):
    """Seeded random mixes of tile-ragged M, N and stage-ragged K (64-k stages, 16-byte k granularity) in every layout,
    including the decode-sized tiles (M <= 64)."""
    test_gemm_layouts(layout, G, M, N, K)


def test_gemm_strided_output_and_operands():
    """Leading dimensions larger than the logical extents (sub-matrix views) and untouched padding."""
    torch = _torch()
    G, M, N, K = 2, 136, 72, 88
    lda, ldb, ldc = K + 16, K + 8, N + 24
    d = I.make_gemm_inputs(G, M, N, K, seed=5)
    a = np.zeros((G, M, lda), np.uint16)
    b = np.zeros((G, N, ldb), np.uint16)
    a[:, :, :K], b[:, :, :K] = d["a"], d["b"]
    a[:, :, K:], b[:, :, K:] = 0x7FC0, 0x7FC0                     # NaN in the padding must never be read into C
    c = torch.zeros((G, M, ldc), dtype=torch.bfloat16, device="cuda")
    B.gemm_bf16(B.to_device(a), B.to_device(b), c, B.GEMM_NT, G, M, N, K, lda, ldb, ldc, M * lda, N * ldb, M * ldc)
    torch.cuda.synchronize()
    got = bits_to_f64(B.to_host_bits(c))
    want = np.einsum("gmk,gnk->gmn", O.widen_bf16(d["a"]), O.widen_bf16(d["b"]))
    assert_close(got[:, :, :N], want, "gemm strided", tol=5e-3)
    assert np.all(got[:, :, N:] == 0.0)


# ------------------------------------------------------------------------------------------ activation, exhaustive
def test_gelu_and_derivative_on_every_bf16_input():
    """The fused epilogues evaluate GELU and its derivative on the bf16-rounded pre-activation, so both are functions
    of a 16-bit input: run all 65 280 finite bf16 values through the block (one rank, no sync, X = value in channel
    0, A = e_0 rows so that P = value; dR' = e_0, dX' = 0, B row 0 = 1 so that dY = 1 and dP = gelu'(P)) and compare
    element by element with the oracle's erf forms."""
    torch = _torch()
    h, fr = 8, 8
    bits = np.arange(65536, dtype=np.uint32)
    finite = ((bits >> 7) & 0xFF) != 0xFF
    vals = bits[finite].astype(np.uint16)
    n = vals.size
    cfg = I.BlockConfig("act", I.KIND_MLP_GELU, I.NORM_LAYERNORM, h=h, T=1, p=0.0, batch=1, seq=n, ffn=fr)
    one = int(I.f32_to_bf16_bits(np.array([1.0], dtype=np.float32))[0])
    X = np.zeros((1, n, h), dtype=np.uint16)
    X[0, :, 0] = vals
    A = np.zeros((1, fr, h), dtype=np.uint16)
    A[0, :, 0] = one
    Bw = np.zeros((1, h, fr), dtype=np.uint16)
    Bw[0, 0, :] = one
    gamma = np.full(h, one, dtype=np.uint16)
    beta = np.zeros(h, dtype=np.uint16)
    R = np.zeros((1, n, h), dtype=np.uint16)
    dXo = np.zeros((1, n, h), dtype=np.uint16)
    dRo = np.zeros((1, n, h), dtype=np.uint16)
    dRo[0, :, 0] = one
    desc = B.make_desc(cfg)
    w0, w1, g, b = B.to_device(A), B.to_device(Bw), B.to_device(gamma), B.to_device(beta)
    x, r = B.to_device(X), B.to_device(R)
    r_out, x_out = torch.empty_like(x), torch.empty_like(x)
    ws = torch.zeros(B.workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    B.block_fwd(desc, [w0, w1, g, b], x, r, r_out, x_out, ws)
    dx, dr = torch.empty_like(x), torch.empty_like(x)
    dw0, dw1 = torch.empty_like(w0), torch.empty_like(w1)
    dgamma = torch.empty(h, dtype=torch.float32, device="cuda")
    dbeta = torch.empty(h, dtype=torch.float32, device="cuda")
    B.block_bwd(desc, [w0, w1, g, b], x, r_out, ws, B.to_device(dXo), B.to_device(dRo), dx, dr, [dw0, dw1], dgamma, dbeta)
    torch.cuda.synchronize()
    L = B.workspace_layout(desc)

    def ws_bits(off, nbytes):
        return ws[off:off + nbytes].view(torch.int16).cpu().numpy().view(np.uint16).reshape(n, fr)

    P, Y, dP = ws_bits(L.off_P, L.bytes_P), ws_bits(L.off_Y, L.bytes_Y), ws_bits(L.off_dP, L.bytes_dP)
    v = bits_to_f64(vals)
    # -0.0 * 1 + 0 * 0 ... accumulates to +0.0: compare values, not bits, for the zero inputs
    assert np.array_equal(bits_to_f64(P[:, 0]), v), "pre-activation must be the input value itself"
    for j in range(1, fr):
        assert np.array_equal(P[:, j], P[:, 0]) and np.array_equal(Y[:, j], Y[:, 0]) and np.array_equal(dP[:, j], dP[:, 0])
    y, want = bits_to_f64(Y[:, 0]), O.gelu(v)
    # bf16 rounding of the result (2^-9 relative) + the evaluation's own error (2.5e-4 relative in the lower tail
    # down to |x| = 5.5, below 1e-7 absolute beyond)
    bound = 2.0 ** -8 * np.abs(want) + 1e-7
    bad = np.abs(y - want) > bound
    assert not bad.any(), "gelu: %d inputs off, worst at x = %r" % (bad.sum(), v[np.argmax(np.abs(y - want) - bound)])
    dy, dwant = bits_to_f64(dP[:, 0]), O.gelu_grad(v)
    dbound = 2.0 ** -8 * np.abs(dwant) + 3e-5
    dbad = np.abs(dy - dwant) > dbound
    assert not dbad.any(), "gelu': %d inputs off, worst at x = %r" % (dbad.sum(), v[np.argmax(np.abs(dy - dwant) - dbound)])
