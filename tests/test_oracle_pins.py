"""Pins for the CPU oracle: each oracle function is checked against something other than itself --
values the paper prints, closed forms, invariants, brute-force Python loops on tiny shapes and
central finite differences in fp64.  CPU only."""
import math
import os

import numpy as np
import pytest

from oracle import caat_oracle as O
from paper_2506_19645_amd import inputs as I
from tests.util import make_inputs, hs_of

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed=0):
    return np.random.default_rng(seed)


# --------------------------------------------------------------------------- channel selection
def test_shared_channels_paper_examples():
    """Sec. 5.2 / Sec. 3 worked examples stored in tests/golden/shared_channels.txt."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "shared_channels.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) >= 5
    for h, p, hs, mult16, _ in rows:
        got = O.shared_channels(int(h), float(p))
        assert got == int(hs)
        assert (got % 16 == 0) == bool(int(mult16))


def test_shared_channels_floor_and_range():
    assert O.shared_channels(768, 0.3) == 230          # 230.4 -> floor
    assert O.shared_channels(768, 0.5) == 384
    assert O.shared_channels(10, 0.99) == 9
    for bad in (-0.1, 1.0001, float("nan")):
        with pytest.raises(ValueError):
            O.shared_channels(16, bad)


# --------------------------------------------------------------------------- partial channel-reduce (Eq. A3)
def _pcr_bruteforce(Zt, hs, scale):
    T, n, h = Zt.shape
    Z = [[[0.0] * h for _ in range(n)] for _ in range(T)]
    for m in range(T):
        for i in range(n):
            for l in range(h):
                if l < hs:
                    acc = 0.0
                    for mm in range(T):
                        acc += float(Zt[mm, i, l])
                    Z[m][i][l] = acc
                else:
                    Z[m][i][l] = scale * float(Zt[m, i, l])
    return np.array(Z)


@pytest.mark.parametrize("T", [1, 2, 3, 8])
def test_pcr_bruteforce_integer_exact(T):
    h, n = 16, 3
    d = I.make_sync_inputs(T, n, h, seed=T, integer=True)
    Zt = O.widen_bf16(d["Zt"])
    for hs in (0, 1, 7, 8, 9, h - 1, h):
        for scale in (1.0, 2.0):
            got = O.partial_channel_reduce(Zt, hs, scale)
            want = _pcr_bruteforce(Zt, hs, scale)
            assert np.array_equal(got, want), (T, hs, scale)


def test_pcr_p1_is_allreduce_p0_is_identity():
    Zt = _rng(1).standard_normal((4, 5, 12))
    full = O.partial_channel_reduce(Zt, 12)
    for m in range(4):
        np.testing.assert_allclose(full[m], Zt.sum(axis=0), rtol=1e-14, atol=1e-14)   # textbook all-reduce
        assert np.array_equal(full[m], full[0])
    none = O.partial_channel_reduce(Zt, 0)
    assert np.array_equal(none, Zt)                                                   # ensemble limit: bits unchanged


def test_pcr_shared_identical_private_untouched():
    Zt = _rng(2).standard_normal((3, 4, 10))
    Z = O.partial_channel_reduce(Zt, 6)
    for m in range(1, 3):
        assert np.array_equal(Z[m, :, :6], Z[0, :, :6])
    assert np.array_equal(Z[:, :, 6:], Zt[:, :, 6:])
    assert not np.array_equal(Z[0, :, 6:], Z[1, :, 6:])


def test_pcr_self_adjoint():
    """sum_m <PCR(a)_m, b_m> == sum_m <a_m, PCR(b)_m>: the backward reduce is the same operator (Fig. 2b)."""
    r = _rng(3)
    a, b = r.standard_normal((4, 6, 9)), r.standard_normal((4, 6, 9))
    for hs in (0, 4, 9):
        for scale in (1.0, 2.0):
            lhs = (O.partial_channel_reduce(a, hs, scale) * b).sum()
            rhs = (a * O.partial_channel_reduce(b, hs, scale)).sum()
            assert abs(lhs - rhs) <= 1e-11 * (abs(lhs) + 1)


def test_private_channel_scaling_variance():
    """Sec. 4: Var(shared) = T sigma^2, Var(private) = sigma^2; equal after scaling private channels by sqrt(T)."""
    T, n, h, hs = 4, 4000, 32, 16
    Zt = _rng(4).standard_normal((T, n, h)) * 0.7
    Z = O.partial_channel_reduce(Zt, hs, 1.0)
    vs, vp = Z[0, :, :hs].var(), Z[0, :, hs:].var()
    assert abs(vs / vp - T) < 0.15 * T
    Zs = O.partial_channel_reduce(Zt, hs, math.sqrt(T))
    assert abs(Zs[0, :, :hs].var() / Zs[0, :, hs:].var() - 1.0) < 0.1


# --------------------------------------------------------------------------- activations
def _phi_quadrature(x, steps=200001):
    """Standard normal CDF by composite Simpson on [-12, x] (independent of erf)."""
    t = np.linspace(-12.0, x, steps)
    f = np.exp(-0.5 * t * t) / math.sqrt(2 * math.pi)
    hstep = (x + 12.0) / (steps - 1)
    return hstep / 3.0 * (f[0] + f[-1] + 4 * f[1:-1:2].sum() + 2 * f[2:-1:2].sum())


def test_gelu_closed_forms():
    assert O.gelu(np.array(0.0)) == 0.0
    for x in (-3.0, -1.0, -0.3, 0.5, 1.0, 2.5):
        assert abs(float(O.gelu(np.array(x))) - x * _phi_quadrature(x)) < 1e-9
    xs = np.linspace(-6, 6, 101)
    np.testing.assert_allclose(O.gelu(xs) - O.gelu(-xs), xs, atol=1e-13)   # x(Phi(x)+Phi(-x)) = x
    assert abs(float(O.gelu(np.array(1.0))) - 0.8413447460685429) < 1e-12  # Phi(1), textbook value
    assert abs(float(O.gelu(np.array(30.0))) - 30.0) < 1e-12


def test_silu_closed_forms():
    assert abs(float(O.silu(np.array(1.0))) - 1.0 / (1.0 + 1.0 / math.e)) < 1e-15
    assert O.silu(np.array(0.0)) == 0.0
    xs = np.linspace(-8, 8, 101)
    np.testing.assert_allclose(O.silu(xs) - O.silu(-xs), xs, atol=1e-13)   # x(s(x)+s(-x)) = x


@pytest.mark.parametrize("fn,grad", [(O.gelu, O.gelu_grad), (O.silu, O.silu_grad)])
def test_activation_grads_fd(fn, grad):
    xs = np.linspace(-5, 5, 201)
    e = 1e-6
    fd = (fn(xs + e) - fn(xs - e)) / (2 * e)
    np.testing.assert_allclose(grad(xs), fd, atol=1e-8)


# --------------------------------------------------------------------------- norms
def test_layernorm_invariants():
    x = _rng(5).standard_normal((2, 7, 64)) * 3 + 1.5
    ones, zeros = np.ones(64), np.zeros(64)
    y, xhat, rstd = O.norm_fwd(x, ones, zeros, O.LAYERNORM, 0.0)
    np.testing.assert_allclose(y.mean(-1), 0, atol=1e-13)
    np.testing.assert_allclose((y * y).mean(-1), 1, atol=1e-12)
    y2, _, _ = O.norm_fwd(5.0 * x + 11.0, ones, zeros, O.LAYERNORM, 0.0)       # shift/scale invariance
    np.testing.assert_allclose(y2, y, atol=1e-11)
    g, b = _rng(6).standard_normal(64), _rng(7).standard_normal(64)
    y3, _, _ = O.norm_fwd(x, g, b, O.LAYERNORM, 0.0)
    np.testing.assert_allclose(y3, y * g + b, atol=1e-13)                      # affine part
    # eps enters under the square root, added to the biased variance
    row = np.array([[[1.0, 3.0]]])                                              # mean 2, var 1
    y4, _, r4 = O.norm_fwd(row, np.ones(2), np.zeros(2), O.LAYERNORM, 3.0)
    np.testing.assert_allclose(r4, 0.5)
    np.testing.assert_allclose(y4, [[[-0.5, 0.5]]])


def test_rmsnorm_invariants():
    x = _rng(8).standard_normal((2, 5, 48)) * 2 + 0.7
    y, _, _ = O.norm_fwd(x, np.ones(48), None, O.RMSNORM, 0.0)
    np.testing.assert_allclose((y * y).mean(-1), 1, atol=1e-12)
    y2, _, _ = O.norm_fwd(-7.0 * x, np.ones(48), None, O.RMSNORM, 0.0)
    np.testing.assert_allclose(y2, -y, atol=1e-12)
    row = np.array([[[3.0, 4.0]]])                                              # mean square 12.5
    y3, _, r3 = O.norm_fwd(row, np.array([2.0, 1.0]), None, O.RMSNORM, 3.5)     # 1/sqrt(16) = 0.25
    np.testing.assert_allclose(r3, 0.25)
    np.testing.assert_allclose(y3, [[[1.5, 1.0]]])


@pytest.mark.parametrize("kind", [O.LAYERNORM, O.RMSNORM])
def test_norm_bwd_fd(kind):
    r = _rng(9 + kind)
    x = r.standard_normal((2, 3, 10))
    g, b = 1 + 0.1 * r.standard_normal(10), 0.1 * r.standard_normal(10)
    w = r.standard_normal((2, 3, 10))
    eps = 1e-5

    def loss(x_, g_, b_):
        y, _, _ = O.norm_fwd(x_, g_, b_ if kind == O.LAYERNORM else None, kind, eps)
        return (y * w).sum()

    dx, dgm, dbm = O.norm_bwd(w, x, g, kind, eps)
    e = 1e-6
    for idx in [(0, 0, 0), (1, 2, 9), (0, 1, 4)]:
        xp, xm = x.copy(), x.copy()
        xp[idx] += e
        xm[idx] -= e
        assert abs((loss(xp, g, b) - loss(xm, g, b)) / (2 * e) - dx[idx]) < 1e-7
    for j in (0, 5, 9):
        gp, gm = g.copy(), g.copy()
        gp[j] += e
        gm[j] -= e
        assert abs((loss(x, gp, b) - loss(x, gm, b)) / (2 * e) - dgm.sum(0)[j]) < 1e-7
        if kind == O.LAYERNORM:
            bp, bm = b.copy(), b.copy()
            bp[j] += e
            bm[j] -= e
            assert abs((loss(x, g, bp) - loss(x, g, bm)) / (2 * e) - dbm.sum(0)[j]) < 1e-7


# --------------------------------------------------------------------------- MLP block
def _tiny_mlp(swiglu, T=2, n=4, h=16, f=32, seed=0, mode="divergent", p=0.5):
    cfg = I.BlockConfig("tiny", I.KIND_MLP_SWIGLU if swiglu else I.KIND_MLP_GELU,
                        I.NORM_RMSNORM if swiglu else I.NORM_LAYERNORM, h=h, T=T, p=p, batch=1, seq=n, ffn=f)
    d = make_inputs(cfg, seed=seed, mode=mode, weight_std=0.3)
    w = {k: O.widen_bf16(v) for k, v in d.items()}
    return cfg, w


def _naive_matmul(a, b):
    n, k = a.shape
    k2, m = b.shape
    assert k == k2
    out = np.zeros((n, m))
    for i in range(n):
        for j in range(m):
            s = 0.0
            for t in range(k):
                s += a[i, t] * b[t, j]
            out[i, j] = s
    return out


@pytest.mark.parametrize("swiglu", [False, True])
def test_mlp_p1_replicated_equals_dense_block(swiglu):
    """Sum of shards is the full GEMM (Eq. 5, Eq. A2): p=1 with replicated input equals the unsharded MLP."""
    cfg, w = _tiny_mlp(swiglu, T=2, n=3, h=8, f=12, mode="replicated", p=1.0)
    norm = O.RMSNORM if swiglu else O.LAYERNORM
    out = O.mlp_block_fwd(w["X"], w["R"], w, w["gamma"], w.get("beta"), swiglu=swiglu, norm=norm, hs=cfg.h)
    X, R = w["X"][0], w["R"][0]
    Bfull = np.concatenate([w["B"][m].T for m in range(cfg.T)], axis=0)       # [f, h]
    if swiglu:
        Wg = np.concatenate([w["Wg"][m].T for m in range(cfg.T)], axis=1)     # [h, f]
        Wu = np.concatenate([w["Wu"][m].T for m in range(cfg.T)], axis=1)
        pg, pu = _naive_matmul(X, Wg), _naive_matmul(X, Wu)
        Y = np.array([[pg[i, j] / (1 + math.exp(-pg[i, j])) * pu[i, j] for j in range(cfg.ffn)] for i in range(3)])
    else:
        Afull = np.concatenate([w["A"][m].T for m in range(cfg.T)], axis=1)
        pp = _naive_matmul(X, Afull)
        Y = np.array([[0.5 * pp[i, j] * (1 + math.erf(pp[i, j] / math.sqrt(2))) for j in range(cfg.ffn)]
                      for i in range(3)])
    Rp = _naive_matmul(Y, Bfull) + R
    for m in range(cfg.T):
        np.testing.assert_allclose(out["Rp"][m], Rp, rtol=1e-12, atol=1e-12)
        assert np.array_equal(out["Xp"][m], out["Xp"][0])
    # dense norm written out by hand
    if swiglu:
        want = Rp / np.sqrt((Rp ** 2).mean(-1, keepdims=True) + 1e-5) * w["gamma"]
    else:
        mu = Rp.mean(-1, keepdims=True)
        want = (Rp - mu) / np.sqrt(((Rp - mu) ** 2).mean(-1, keepdims=True) + 1e-5) * w["gamma"] + w["beta"]
    np.testing.assert_allclose(out["Xp"][0], want, rtol=1e-12, atol=1e-12)


def test_mlp_two_rank_block_formula():
    """Eq. 8: Z_1 = [Y_1 B_11 + Y_2 B_12, Y_1 B_21], Z_2 = [same, Y_2 B_22] with explicit sub-blocks of B."""
    cfg, w = _tiny_mlp(False, T=2, n=3, h=8, f=12, p=0.5)
    hs = hs_of(cfg)
    out = O.mlp_block_fwd(w["X"], w["R"], w, w["gamma"], w["beta"], swiglu=False, norm=O.LAYERNORM, hs=hs)
    Y1, Y2 = out["Y"]
    B1, B2 = w["B"][0].T, w["B"][1].T           # [f/2, h] row blocks of B held by device 1 and 2
    B11, B21 = B1[:, :hs], B1[:, hs:]
    B12, B22 = B2[:, :hs], B2[:, hs:]
    shared = _naive_matmul(Y1, B11) + _naive_matmul(Y2, B12)
    np.testing.assert_allclose(out["Z"][0], np.concatenate([shared, _naive_matmul(Y1, B21)], 1), atol=1e-12)
    np.testing.assert_allclose(out["Z"][1], np.concatenate([shared, _naive_matmul(Y2, B22)], 1), atol=1e-12)
    # first layer: each device multiplies ITS input by ITS column block (Eq. 6)
    pre = _naive_matmul(w["X"][1], w["A"][1].T)
    np.testing.assert_allclose(out["P"][1], pre, atol=1e-12)


def test_mlp_p0_is_local_partial_sum():
    cfg, w = _tiny_mlp(True, T=3, n=4, h=16, f=48, p=0.0)
    out = O.mlp_block_fwd(w["X"], w["R"], w, w["gamma"], None, swiglu=True, norm=O.RMSNORM, hs=0)
    assert np.array_equal(out["Z"], out["Zt"])
    assert np.array_equal(out["Rp"], w["R"] + out["Zt"])


def _mlp_loss(cfg, w, Wt, Vt, swiglu, hs, scale):
    norm = O.RMSNORM if swiglu else O.LAYERNORM
    out = O.mlp_block_fwd(w["X"], w["R"], w, w["gamma"], w.get("beta"), swiglu=swiglu, norm=norm, hs=hs,
                          private_scale=scale)
    return (out["Xp"] * Wt).sum() + (out["Rp"] * Vt).sum()


@pytest.mark.parametrize("swiglu", [False, True])
@pytest.mark.parametrize("hs,scale", [(0, 1.0), (5, 1.0), (8, math.sqrt(2.0)), (16, 1.0)])
def test_mlp_backward_finite_differences(swiglu, hs, scale):
    """L = sum_m <W_m, X'_m> + <V_m, R'_m>; every gradient vs central differences in fp64."""
    cfg, w = _tiny_mlp(swiglu, T=2, n=4, h=16, f=32, seed=3)
    norm = O.RMSNORM if swiglu else O.LAYERNORM
    r = _rng(11)
    Wt, Vt = r.standard_normal(w["X"].shape), r.standard_normal(w["X"].shape)
    fwd = O.mlp_block_fwd(w["X"], w["R"], w, w["gamma"], w.get("beta"), swiglu=swiglu, norm=norm, hs=hs,
                          private_scale=scale)
    g = O.mlp_block_bwd(w["X"], fwd, w, w["gamma"], Wt, Vt, swiglu=swiglu, norm=norm, hs=hs, private_scale=scale)
    names = {"X": "dX", "R": "dR", "B": "dB", "gamma": "dgamma"}
    names.update({"Wg": "dWg", "Wu": "dWu"} if swiglu else {"A": "dA", "beta": "dbeta"})
    e = 1e-6
    for key, gname in names.items():
        arr = w[key]
        flat_idx = r.choice(arr.size, size=min(6, arr.size), replace=False)
        for fi in flat_idx:
            idx = np.unravel_index(fi, arr.shape)
            old = arr[idx]
            arr[idx] = old + e
            lp = _mlp_loss(cfg, w, Wt, Vt, swiglu, hs, scale)
            arr[idx] = old - e
            lm = _mlp_loss(cfg, w, Wt, Vt, swiglu, hs, scale)
            arr[idx] = old
            fd = (lp - lm) / (2 * e)
            assert abs(fd - g[gname][idx]) < 2e-6 * (1 + abs(fd)), (key, idx, fd, g[gname][idx])


def test_dx_not_reduced_and_dr_is_g():
    """No reduce at the column-parallel input (Sec. 4): dX_m depends only on rank m's upstream gradient when hs=0."""
    cfg, w = _tiny_mlp(False, T=2, n=3, h=8, f=12, seed=5)
    r = _rng(12)
    dXo, dRo = r.standard_normal(w["X"].shape), r.standard_normal(w["X"].shape)
    fwd = O.mlp_block_fwd(w["X"], w["R"], w, w["gamma"], w["beta"], swiglu=False, norm=O.LAYERNORM, hs=0)
    g0 = O.mlp_block_bwd(w["X"], fwd, w, w["gamma"], dXo, dRo, swiglu=False, norm=O.LAYERNORM, hs=0)
    dXo2 = dXo.copy()
    dXo2[1] += 1.0
    g1 = O.mlp_block_bwd(w["X"], fwd, w, w["gamma"], dXo2, dRo, swiglu=False, norm=O.LAYERNORM, hs=0)
    assert np.array_equal(g0["dX"][0], g1["dX"][0])
    assert not np.array_equal(g0["dX"][1], g1["dX"][1])


def test_backward_placement_equivalence_full_sync():
    """Sec. 4: with full all-reduce (p=1, replicated inputs) reducing after the norm backward plus summing the
    norm-parameter gradients equals the vanilla order (reduce first, then one norm backward)."""
    cfg, w = _tiny_mlp(False, T=3, n=4, h=12, f=24, mode="replicated", p=1.0, seed=7)
    r = _rng(13)
    dXo = r.standard_normal(w["X"].shape)
    dRo = np.zeros_like(dXo)
    fwd = O.mlp_block_fwd(w["X"], w["R"], w, w["gamma"], w["beta"], swiglu=False, norm=O.LAYERNORM, hs=cfg.h)
    g = O.mlp_block_bwd(w["X"], fwd, w, w["gamma"], dXo, dRo, swiglu=False, norm=O.LAYERNORM, hs=cfg.h)
    # vanilla: sum upstream gradients over ranks first, then one norm backward on the (identical) activations
    dsum = dXo.sum(axis=0, keepdims=True)
    dn, dgam, dbet = O.norm_bwd(dsum, fwd["Rp"][:1], w["gamma"], O.LAYERNORM, 1e-5)
    for m in range(cfg.T):
        np.testing.assert_allclose(g["dZt"][m], dn[0], rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(g["dgamma"], dgam[0], rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(g["dbeta"], dbet[0], rtol=1e-11, atol=1e-12)


# --------------------------------------------------------------------------- attention
def _naive_attention(q, k, v, q_pos0=0):
    sq, d = q.shape
    out = np.zeros((sq, v.shape[1]))
    for i in range(sq):
        last = q_pos0 + i
        sc = [sum(q[i, t] * k[j, t] for t in range(d)) / math.sqrt(d) for j in range(last + 1)]
        mx = max(sc)
        ex = [math.exp(s - mx) for s in sc]
        z = sum(ex)
        for j in range(last + 1):
            out[i] += ex[j] / z * v[j]
    return out


def test_causal_attention_tiny_vs_loops_and_invariants():
    r = _rng(14)
    q, k, v = r.standard_normal((6, 4)), r.standard_normal((6, 4)), r.standard_normal((6, 4))
    got = O.causal_attention(q, k, v)
    np.testing.assert_allclose(got, _naive_attention(q, k, v), atol=1e-13)
    np.testing.assert_allclose(got[0], v[0], atol=1e-14)                       # first token sees only itself
    np.testing.assert_allclose(O.causal_attention(q, k, np.ones_like(v)), 1.0, atol=1e-14)  # softmax rows sum to 1
    k2, v2 = k.copy(), v.copy()
    k2[4:] += 5.0
    v2[4:] -= 3.0
    np.testing.assert_allclose(O.causal_attention(q, k2, v2)[:4], got[:4], atol=1e-14)      # causality


def test_rope_properties():
    r = _rng(15)
    d = 8
    x = r.standard_normal((5, d))
    assert np.array_equal(O.rope(x, np.zeros(5), 10000.0), x)                  # position 0 is the identity
    y = O.rope(x, np.arange(5), 10000.0)
    np.testing.assert_allclose((y ** 2).sum(-1), (x ** 2).sum(-1), rtol=1e-13)  # rotation keeps the norm
    # pair (0, d/2) rotates by pos * base^0 = pos radians
    e0 = np.zeros((1, d))
    e0[0, 0] = 1.0
    y0 = O.rope(e0, np.array([1.0]), 10000.0)
    np.testing.assert_allclose([y0[0, 0], y0[0, d // 2]], [math.cos(1.0), math.sin(1.0)], atol=1e-15)
    # pair (1, 1+d/2) rotates by pos * base^(-2/d)
    e1 = np.zeros((1, d))
    e1[0, 1] = 1.0
    y1 = O.rope(e1, np.array([3.0]), 10000.0)
    th = 3.0 * 10000.0 ** (-2.0 / d)
    np.testing.assert_allclose([y1[0, 1], y1[0, 1 + d // 2]], [math.cos(th), math.sin(th)], atol=1e-15)
    # relative-position property: scores depend on position differences only
    q, k = r.standard_normal((5, d)), r.standard_normal((5, d))
    s0 = O.rope(q, np.arange(5), 10000.0) @ O.rope(k, np.arange(5), 10000.0).T
    s7 = O.rope(q, np.arange(5) + 7, 10000.0) @ O.rope(k, np.arange(5) + 7, 10000.0).T
    np.testing.assert_allclose(s0, s7, atol=1e-12)


def _tiny_attn(T=2, batch=2, seq=5, heads=4, d=4, p=0.5, seed=0):
    cfg = I.BlockConfig("tinyattn", I.KIND_ATTN, I.NORM_RMSNORM, h=heads * d, T=T, p=p, batch=batch, seq=seq,
                        n_heads=heads, head_dim=d)
    dd = make_inputs(cfg, seed=seed, weight_std=0.3)
    return cfg, {k: O.widen_bf16(v) for k, v in dd.items()}


def test_attention_block_tiny_vs_loops():
    cfg, w = _tiny_attn()
    hpr, d, hd = cfg.n_heads // cfg.T, cfg.head_dim, cfg.hd_r
    out = O.attn_block_fwd(w["X"], w["R"], w["Wqkv"], w["Wo"], w["gamma"], None, batch=cfg.batch, seq=cfg.seq,
                           heads_per_rank=hpr, head_dim=d, norm=O.RMSNORM, hs=hs_of(cfg))
    half = d // 2
    for m in range(cfg.T):
        qkv = _naive_matmul(w["X"][m], w["Wqkv"][m].T)
        Hm = np.zeros((cfg.tokens, hd))
        for b in range(cfg.batch):
            for a in range(hpr):
                rows = range(b * cfg.seq, (b + 1) * cfg.seq)
                q = np.zeros((cfg.seq, d))
                k = np.zeros((cfg.seq, d))
                v = np.zeros((cfg.seq, d))
                for t, row in enumerate(rows):
                    for j in range(half):
                        th = t * 10000.0 ** (-2.0 * j / d)
                        c, s = math.cos(th), math.sin(th)
                        for dst, off in ((q, 0), (k, hd)):
                            x1, x2 = qkv[row, off + a * d + j], qkv[row, off + a * d + j + half]
                            dst[t, j] = x1 * c - x2 * s
                            dst[t, j + half] = x2 * c + x1 * s
                    v[t] = qkv[row, 2 * hd + a * d:2 * hd + (a + 1) * d]
                Hm[b * cfg.seq:(b + 1) * cfg.seq, a * d:(a + 1) * d] = _naive_attention(q, k, v)
        np.testing.assert_allclose(out["H"][m], Hm, atol=1e-12)
        np.testing.assert_allclose(out["Zt"][m], _naive_matmul(Hm, w["Wo"][m].T), atol=1e-12)
    # Eq. A5 case split on the attention output
    np.testing.assert_allclose(out["Z"][0, :, :hs_of(cfg)], out["Zt"][:, :, :hs_of(cfg)].sum(0), atol=1e-13)
    assert np.array_equal(out["Z"][:, :, hs_of(cfg):], out["Zt"][:, :, hs_of(cfg):])


def test_attention_block_sequences_independent_and_causal():
    cfg, w = _tiny_attn(batch=2, seq=6)
    kw = dict(batch=cfg.batch, seq=cfg.seq, heads_per_rank=cfg.n_heads // cfg.T, head_dim=cfg.head_dim,
              norm=O.RMSNORM, hs=hs_of(cfg))
    a = O.attn_block_fwd(w["X"], w["R"], w["Wqkv"], w["Wo"], w["gamma"], None, **kw)
    X2 = w["X"].copy()
    X2[:, 6 + 4:] += 1.0       # perturb the tail of sequence 1 only
    b = O.attn_block_fwd(X2, w["R"], w["Wqkv"], w["Wo"], w["gamma"], None, **kw)
    np.testing.assert_allclose(a["Rp"][:, :6 + 4], b["Rp"][:, :6 + 4], atol=1e-14)
    assert not np.allclose(a["Rp"][:, 6 + 4:], b["Rp"][:, 6 + 4:])


# --------------------------------------------------------------------------- attention backward
def test_rope_adjoint_is_transpose_and_inverse():
    r = _rng(21)
    d, s = 8, 6
    x, y = r.standard_normal((s, d)), r.standard_normal((s, d))
    pos = np.arange(s) + 3
    # <rope(x), y> = <x, rope_adjoint(y)> (transpose), and the rotation is orthogonal so adjoint = inverse
    lhs = (O.rope(x, pos, 10000.0) * y).sum()
    rhs = (x * O.rope_adjoint(y, pos, 10000.0)).sum()
    assert abs(lhs - rhs) < 1e-12
    np.testing.assert_allclose(O.rope_adjoint(O.rope(x, pos, 10000.0), pos, 10000.0), x, atol=1e-14)


def _softmax_jacobian_attention_bwd(q, k, v, dO):
    """Attention gradient with the softmax Jacobian written entry by entry (python loops)."""
    sq, d = q.shape
    dq, dk, dv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    for i in range(sq):
        sc = np.array([q[i] @ k[j] / math.sqrt(d) for j in range(i + 1)])
        pr = np.exp(sc - sc.max())
        pr /= pr.sum()
        dp = np.array([dO[i] @ v[j] for j in range(i + 1)])
        for j in range(i + 1):
            dv[j] += pr[j] * dO[i]
            ds = sum(dp[t] * pr[t] * ((1.0 if t == j else 0.0) - pr[j]) for t in range(i + 1))
            dq[i] += ds * k[j] / math.sqrt(d)
            dk[j] += ds * q[i] / math.sqrt(d)
    return dq, dk, dv


def test_causal_attention_bwd_vs_jacobian_loops_and_fd():
    r = _rng(22)
    sq, d = 6, 4
    q, k, v, dO = (r.standard_normal((sq, d)) for _ in range(4))
    dq, dk, dv = O.causal_attention_bwd(q, k, v, dO)
    jq, jk, jv = _softmax_jacobian_attention_bwd(q, k, v, dO)
    np.testing.assert_allclose(dq, jq, atol=1e-13)
    np.testing.assert_allclose(dk, jk, atol=1e-13)
    np.testing.assert_allclose(dv, jv, atol=1e-13)
    # central differences of L = <dO, attention(q,k,v)>
    e = 1e-6
    for arr, grad in ((q, dq), (k, dk), (v, dv)):
        for idx in [(0, 0), (2, 3), (5, 1), (3, 2)]:
            old = arr[idx]
            arr[idx] = old + e
            lp = (O.causal_attention(q, k, v) * dO).sum()
            arr[idx] = old - e
            lm = (O.causal_attention(q, k, v) * dO).sum()
            arr[idx] = old
            assert abs((lp - lm) / (2 * e) - grad[idx]) < 1e-8
    # causality of the gradient: the last key / value only receives gradient from the last query
    dO2 = dO.copy()
    dO2[:sq - 1] = 0.0
    _, dk2, dv2 = O.causal_attention_bwd(q, k, v, dO2)
    np.testing.assert_allclose(dk2[sq - 1], dk[sq - 1], atol=1e-14)
    np.testing.assert_allclose(dv2[sq - 1], dv[sq - 1], atol=1e-14)
    # softmax rows sum to one => a constant added to all values moves O by that constant: sum_j dv_j = sum_i dO_i
    np.testing.assert_allclose(dv.sum(0), dO.sum(0), atol=1e-13)


def _attn_loss(cfg, w, Wt, Vt, hs, scale, norm):
    out = O.attn_block_fwd(w["X"], w["R"], w["Wqkv"], w["Wo"], w["gamma"], w.get("beta"), batch=cfg.batch,
                           seq=cfg.seq, heads_per_rank=cfg.n_heads // cfg.T, head_dim=cfg.head_dim, norm=norm,
                           hs=hs, private_scale=scale)
    return (out["Xp"] * Wt).sum() + (out["Rp"] * Vt).sum()


@pytest.mark.parametrize("hs,scale", [(0, 1.0), (5, 1.0), (8, math.sqrt(2.0)), (16, 1.0)])
def test_attention_block_backward_finite_differences(hs, scale):
    """L = sum_m <W_m, X'_m> + <V_m, R'_m>; every gradient of the attention block vs central differences."""
    cfg, w = _tiny_attn(T=2, batch=2, seq=5, heads=4, d=4, seed=4)
    r = _rng(23)
    Wt, Vt = r.standard_normal(w["X"].shape), r.standard_normal(w["X"].shape)
    kw = dict(batch=cfg.batch, seq=cfg.seq, heads_per_rank=cfg.n_heads // cfg.T, head_dim=cfg.head_dim,
              norm=O.RMSNORM, hs=hs, private_scale=scale)
    fwd = O.attn_block_fwd(w["X"], w["R"], w["Wqkv"], w["Wo"], w["gamma"], None, **kw)
    g = O.attn_block_bwd(w["X"], fwd, w["Wqkv"], w["Wo"], w["gamma"], Wt, Vt, **kw)
    e = 1e-6
    for key, gname in {"X": "dX", "R": "dR", "Wqkv": "dWqkv", "Wo": "dWo", "gamma": "dgamma"}.items():
        arr = w[key]
        for fi in r.choice(arr.size, size=min(8, arr.size), replace=False):
            idx = np.unravel_index(fi, arr.shape)
            old = arr[idx]
            arr[idx] = old + e
            lp = _attn_loss(cfg, w, Wt, Vt, hs, scale, O.RMSNORM)
            arr[idx] = old - e
            lm = _attn_loss(cfg, w, Wt, Vt, hs, scale, O.RMSNORM)
            arr[idx] = old
            fd = (lp - lm) / (2 * e)
            assert abs(fd - g[gname][idx]) < 2e-6 * (1 + abs(fd)), (key, idx, fd, g[gname][idx])


def test_attention_backward_no_reduce_at_input_and_sequences_independent():
    """dX_m depends only on rank m's upstream gradient when hs = 0 (Sec. 4: no reduce at the column-parallel input),
    and a gradient entering sequence 1 leaves sequence 0's dX untouched."""
    cfg, w = _tiny_attn(T=2, batch=2, seq=4, heads=4, d=4, seed=6)
    r = _rng(24)
    dXo, dRo = r.standard_normal(w["X"].shape), r.standard_normal(w["X"].shape)
    kw = dict(batch=cfg.batch, seq=cfg.seq, heads_per_rank=cfg.n_heads // cfg.T, head_dim=cfg.head_dim,
              norm=O.RMSNORM, hs=0)
    fwd = O.attn_block_fwd(w["X"], w["R"], w["Wqkv"], w["Wo"], w["gamma"], None, **kw)
    g0 = O.attn_block_bwd(w["X"], fwd, w["Wqkv"], w["Wo"], w["gamma"], dXo, dRo, **kw)
    d2 = dXo.copy()
    d2[1, cfg.seq:] += 1.0          # rank 1, sequence 1 only
    g1 = O.attn_block_bwd(w["X"], fwd, w["Wqkv"], w["Wo"], w["gamma"], d2, dRo, **kw)
    assert np.array_equal(g0["dX"][0], g1["dX"][0])
    assert np.array_equal(g0["dX"][1, :cfg.seq], g1["dX"][1, :cfg.seq])
    assert not np.array_equal(g0["dX"][1, cfg.seq:], g1["dX"][1, cfg.seq:])


# --------------------------------------------------------------------------- decode layer
def test_decode_equals_last_row_of_prefill():
    """The decode step over a cache of L rotated keys equals row L of a causal prefill over L+1 tokens."""
    T, b, heads, d, L = 2, 2, 4, 4, 5
    h, f = heads * d, 24
    cfg = I.BlockConfig("tinydec", I.KIND_DECODE, I.NORM_RMSNORM, h=h, T=T, p=0.5, batch=b, seq=1, ffn=f,
                        n_heads=heads, head_dim=d, kv_len=L)
    dd = make_inputs(cfg, seed=2, weight_std=0.3)
    w = {k: O.widen_bf16(v) for k, v in dd.items()}
    hpr = heads // T
    # A prefill over L+1 tokens per sequence with random normalised inputs; its K, V fill the cache.
    r = _rng(16)
    Rfull = r.standard_normal((T, b * (L + 1), h))
    X1full, _, _ = O.norm_fwd(Rfull, w["gamma_attn"], None, O.RMSNORM, 1e-5)
    pre = O.attn_block_fwd(X1full, Rfull, w["Wqkv"], w["Wo"], w["gamma"], None, batch=b, seq=L + 1,
                           heads_per_rank=hpr, head_dim=d, norm=O.RMSNORM, hs=hs_of(cfg))
    Kc = np.zeros((T, b, hpr, L + 1, d))
    Vc = np.zeros_like(Kc)
    Kc[:, :, :, :L] = pre["K"][:, :, :, :L]
    Vc[:, :, :, :L] = pre["V"][:, :, :, :L]
    last = [s * (L + 1) + L for s in range(b)]
    Rlast = Rfull[:, last]
    dec = O.decode_layer_fwd(Rlast, w, Kc, Vc, kv_len=L, heads_per_rank=hpr, head_dim=d, hs=hs_of(cfg))
    np.testing.assert_allclose(dec["R1"], pre["Rp"][:, last], atol=1e-12)
    np.testing.assert_allclose(dec["X2"], pre["Xp"][:, last], atol=1e-12)
    np.testing.assert_allclose(dec["k_new"], pre["K"][:, :, :, L], atol=1e-13)
    np.testing.assert_allclose(dec["v_new"], pre["V"][:, :, :, L], atol=1e-13)
    # the MLP half equals the MLP block applied to (X2, R1)
    mlp = O.mlp_block_fwd(dec["X2"], dec["R1"], w, w["gamma"], None, swiglu=True, norm=O.RMSNORM, hs=hs_of(cfg))
    np.testing.assert_allclose(dec["R2"], mlp["Rp"], atol=1e-13)


# --------------------------------------------------------------------------- grouped-query attention
def _tiny_gqa(T=2, batch=2, seq=5, heads=8, kv_heads=4, d=4, p=0.5, seed=9, kind=I.KIND_ATTN, ffn=0, kv_len=0):
    cfg = I.BlockConfig("tinygqa", kind, I.NORM_RMSNORM, h=heads * d, T=T, p=p, batch=batch, seq=seq, ffn=ffn,
                        n_heads=heads, head_dim=d, n_kv_heads=kv_heads, kv_len=kv_len)
    dd = make_inputs(cfg, seed=seed, weight_std=0.3)
    return cfg, {k: O.widen_bf16(v) for k, v in dd.items()}


def _expand_kv_rows(Wqkv, hpr, kvpr, d):
    """Multi-head projection shard that repeats every key / value head once per query head of its group."""
    grp, hd, kvd = hpr // kvpr, hpr * d, kvpr * d
    q = Wqkv[:, :hd]
    k = Wqkv[:, hd:hd + kvd].reshape(Wqkv.shape[0], kvpr, d, -1)
    v = Wqkv[:, hd + kvd:].reshape(Wqkv.shape[0], kvpr, d, -1)
    rep = lambda t: np.repeat(t, grp, axis=1).reshape(Wqkv.shape[0], hd, -1)
    return np.concatenate([q, rep(k), rep(v)], axis=1)


def test_gqa_equals_mha_with_repeated_kv_heads_forward_and_backward():
    """Grouped-query attention is multi-head attention whose key / value projections are tied within a group: the
    forward equals the (already pinned) multi-head block with the tied rows repeated, and the gradient of a tied
    row is the sum of the gradients of its copies."""
    cfg, w = _tiny_gqa()
    hpr, kvpr, d = cfg.n_heads // cfg.T, cfg.kv_heads // cfg.T, cfg.head_dim
    grp, hd, kvd = hpr // kvpr, hpr * d, kvpr * d
    kw = dict(batch=cfg.batch, seq=cfg.seq, heads_per_rank=hpr, head_dim=d, norm=O.RMSNORM, hs=hs_of(cfg))
    r = _rng(31)
    dXo, dRo = r.standard_normal(w["X"].shape), r.standard_normal(w["X"].shape)
    fg = O.attn_block_fwd(w["X"], w["R"], w["Wqkv"], w["Wo"], w["gamma"], None, kv_heads_per_rank=kvpr, **kw)
    gg = O.attn_block_bwd(w["X"], fg, w["Wqkv"], w["Wo"], w["gamma"], dXo, dRo, kv_heads_per_rank=kvpr, **kw)
    Wm = _expand_kv_rows(w["Wqkv"], hpr, kvpr, d)
    fm = O.attn_block_fwd(w["X"], w["R"], Wm, w["Wo"], w["gamma"], None, **kw)
    gm = O.attn_block_bwd(w["X"], fm, Wm, w["Wo"], w["gamma"], dXo, dRo, **kw)
    for name in ("H", "Rp", "Xp"):
        np.testing.assert_allclose(fg[name], fm[name], atol=1e-12)
    for name in ("dX", "dR", "dWo", "dgamma"):
        np.testing.assert_allclose(gg[name], gm[name], atol=1e-11)
    T = cfg.T
    np.testing.assert_allclose(gg["dWqkv"][:, :hd], gm["dWqkv"][:, :hd], atol=1e-11)
    dk_m = gm["dWqkv"][:, hd:2 * hd].reshape(T, kvpr, grp, d, -1).sum(axis=2).reshape(T, kvd, -1)
    dv_m = gm["dWqkv"][:, 2 * hd:].reshape(T, kvpr, grp, d, -1).sum(axis=2).reshape(T, kvd, -1)
    np.testing.assert_allclose(gg["dWqkv"][:, hd:hd + kvd], dk_m, atol=1e-11)
    np.testing.assert_allclose(gg["dWqkv"][:, hd + kvd:], dv_m, atol=1e-11)


def test_gqa_decode_equals_last_row_of_prefill():
    L = 4
    cfg, w = _tiny_gqa(T=2, batch=2, seq=L + 1, heads=8, kv_heads=4, d=4, kind=I.KIND_PREFILL, ffn=24)
    hpr, kvpr, d = cfg.n_heads // cfg.T, cfg.kv_heads // cfg.T, cfg.head_dim
    pre = O.prefill_layer_fwd(w["R"], w, batch=cfg.batch, seq=cfg.seq, heads_per_rank=hpr, head_dim=d, hs=hs_of(cfg),
                              kv_heads_per_rank=kvpr)
    assert pre["K"].shape == (cfg.T, cfg.batch, kvpr, L + 1, d)
    Kc = np.zeros((cfg.T, cfg.batch, kvpr, L + 1, d))
    Vc = np.zeros_like(Kc)
    Kc[:, :, :, :L] = pre["K"][:, :, :, :L]
    Vc[:, :, :, :L] = pre["V"][:, :, :, :L]
    last = [s * (L + 1) + L for s in range(cfg.batch)]
    dec = O.decode_layer_fwd(w["R"][:, last], w, Kc, Vc, kv_len=L, heads_per_rank=hpr, head_dim=d, hs=hs_of(cfg),
                             kv_heads_per_rank=kvpr)
    np.testing.assert_allclose(dec["R2"], pre["R2"][:, last], atol=1e-12)
    np.testing.assert_allclose(dec["k_new"], pre["K"][:, :, :, L], atol=1e-13)


# --------------------------------------------------------------------------- prefill layer
def _tiny_prefill(T=2, b=2, heads=4, d=4, seq=6, f=24, p=0.5, seed=3, mode="divergent"):
    cfg = I.BlockConfig("tinypre", I.KIND_PREFILL, I.NORM_RMSNORM, h=heads * d, T=T, p=p, batch=b, seq=seq, ffn=f,
                        n_heads=heads, head_dim=d)
    dd = make_inputs(cfg, seed=seed, weight_std=0.3, mode=mode)
    return cfg, {k: O.widen_bf16(v) for k, v in dd.items()}


def test_prefill_layer_last_row_equals_decode_step():
    """A prompt of L+1 tokens through the prefill layer gives, in its last row, what the decode step gives for token
    L over the cache that the first L prompt tokens left (same weights): both halves of the layer, R1 and R2."""
    L = 5
    cfg, w = _tiny_prefill(seq=L + 1)
    hpr, d = cfg.n_heads // cfg.T, cfg.head_dim
    pre = O.prefill_layer_fwd(w["R"], w, batch=cfg.batch, seq=cfg.seq, heads_per_rank=hpr, head_dim=d, hs=hs_of(cfg))
    Kc = np.zeros((cfg.T, cfg.batch, hpr, L + 1, d))
    Vc = np.zeros_like(Kc)
    Kc[:, :, :, :L] = pre["K"][:, :, :, :L]
    Vc[:, :, :, :L] = pre["V"][:, :, :, :L]
    last = [s * (L + 1) + L for s in range(cfg.batch)]
    dec = O.decode_layer_fwd(w["R"][:, last], w, Kc, Vc, kv_len=L, heads_per_rank=hpr, head_dim=d, hs=hs_of(cfg))
    np.testing.assert_allclose(dec["R1"], pre["R1"][:, last], atol=1e-12)
    np.testing.assert_allclose(dec["R2"], pre["R2"][:, last], atol=1e-12)
    np.testing.assert_allclose(dec["k_new"], pre["K"][:, :, :, L], atol=1e-13)
    np.testing.assert_allclose(dec["v_new"], pre["V"][:, :, :, L], atol=1e-13)


@pytest.mark.parametrize("p", [0.0, 0.5, 0.3])
def test_layer_private_scale_equals_prescaled_private_weight_rows(p):
    """Private channel scaling (Sec. 4) multiplies a row-parallel output's private channels by a constant before the
    residual add, so a layer with scale c must equal the SAME layer at scale 1 whose row-parallel weights Wo and B have
    their private OUTPUT rows (l >= hs) multiplied by c beforehand -- in both halves of the layer, for the prefill and
    for the decode function -- and must differ from the unscaled layer.  At p = 0 every row is private: the whole of
    Wo and B is pre-multiplied.  Decode must still equal the last prefill row with the scale on."""
    L = 5
    cfg, w = _tiny_prefill(seq=L + 1, p=p, seed=13)
    T, hpr, d = cfg.T, cfg.n_heads // cfg.T, cfg.head_dim
    hs = hs_of(cfg)
    c = math.sqrt(T)
    kw = dict(heads_per_rank=hpr, head_dim=d, hs=hs)
    pre_c = O.prefill_layer_fwd(w["R"], w, batch=cfg.batch, seq=cfg.seq, private_scale=c, **kw)
    w2 = dict(w)
    w2["Wo"], w2["B"] = w["Wo"].copy(), w["B"].copy()
    w2["Wo"][:, hs:, :] *= c            # [T][h out][hd_r in]: output rows hs.. are the private channels
    w2["B"][:, hs:, :] *= c
    pre_w = O.prefill_layer_fwd(w["R"], w2, batch=cfg.batch, seq=cfg.seq, private_scale=1.0, **kw)
    pre_1 = O.prefill_layer_fwd(w["R"], w, batch=cfg.batch, seq=cfg.seq, private_scale=1.0, **kw)
    for name in ("R1", "X2", "R2"):
        np.testing.assert_allclose(pre_c[name], pre_w[name], atol=1e-12)
        assert np.abs(pre_c[name] - pre_1[name]).max() > 1e-3, name
    # the two halves separately: R1 - R is the scaled attention output, R2 - R1 the scaled MLP output
    for a, b in (("R1", None), ("R2", "R1")):
        zc = pre_c[a] - (w["R"] if b is None else pre_c[b])
        z1_in = pre_c["Zt"] if b is None else pre_c["Zt2"]
        np.testing.assert_allclose(zc[:, :, hs:], c * z1_in[:, :, hs:], atol=1e-12)
        np.testing.assert_allclose(zc[:, :, :hs], np.broadcast_to(z1_in[:, :, :hs].sum(0), zc[:, :, :hs].shape), atol=1e-12)
    # decode over the cache of the first L tokens, scale on: last prefill row; and the pre-scaled-weights identity
    Kc = np.zeros((T, cfg.batch, hpr, L + 1, d))
    Vc = np.zeros_like(Kc)
    Kc[:, :, :, :L] = pre_c["K"][:, :, :, :L]
    Vc[:, :, :, :L] = pre_c["V"][:, :, :, :L]
    last = [s * (L + 1) + L for s in range(cfg.batch)]
    dec_c = O.decode_layer_fwd(w["R"][:, last], w, Kc, Vc, kv_len=L, private_scale=c, **kw)
    dec_w = O.decode_layer_fwd(w["R"][:, last], w2, Kc, Vc, kv_len=L, private_scale=1.0, **kw)
    dec_1 = O.decode_layer_fwd(w["R"][:, last], w, Kc, Vc, kv_len=L, private_scale=1.0, **kw)
    for name in ("R1", "X2", "R2"):
        np.testing.assert_allclose(dec_c[name], dec_w[name], atol=1e-12)
        np.testing.assert_allclose(dec_c[name], pre_c[name][:, last], atol=1e-12)
        assert np.abs(dec_c[name] - dec_1[name]).max() > 1e-3, name
    # each half on its own: a mutation that drops the scale in only ONE half must not hide behind the other
    np.testing.assert_allclose((dec_c["R2"] - dec_c["R1"])[:, :, hs:], c * dec_c["Zt2"][:, :, hs:], atol=1e-12)
    np.testing.assert_allclose((dec_c["R1"] - w["R"][:, last])[:, :, hs:], c * dec_c["Zt"][:, :, hs:], atol=1e-12)


def test_prefill_layer_p1_replicated_equals_dense_llama_layer():
    """p = 1 with replicated inputs is ordinary tensor parallelism, so every rank's output equals the dense layer with
    the shards concatenated; the dense layer is written here independently (complex-number RoPE, per-head loops)."""
    cfg, w = _tiny_prefill(T=2, b=1, heads=4, d=4, seq=5, f=24, p=1.0, seed=8, mode="replicated")
    T, h, d, s = cfg.T, cfg.h, cfg.head_dim, cfg.seq
    hpr, hd = cfg.n_heads // T, cfg.hd_r
    out = O.prefill_layer_fwd(w["R"], w, batch=1, seq=s, heads_per_rank=hpr, head_dim=d, hs=hs_of(cfg))
    x = w["R"][0]

    def rms(v, g):
        return v / np.sqrt((v * v).mean(-1, keepdims=True) + 1e-5) * g

    x1 = rms(x, w["gamma_attn"])
    att = np.zeros_like(x)
    for m in range(T):
        qkv = x1 @ w["Wqkv"][m].T
        for a in range(hpr):
            def rot(t):
                z = (t[:, :d // 2] + 1j * t[:, d // 2:]) * np.exp(
                    1j * np.arange(s)[:, None] * 10000.0 ** (-2.0 * np.arange(d // 2) / d)[None, :])
                return np.concatenate([z.real, z.imag], axis=1)
            q, k = rot(qkv[:, a * d:(a + 1) * d]), rot(qkv[:, hd + a * d:hd + (a + 1) * d])
            v = qkv[:, 2 * hd + a * d:2 * hd + (a + 1) * d]
            att += _naive_attention(q, k, v) @ w["Wo"][m][:, a * d:(a + 1) * d].T
    r1 = x + att
    x2 = rms(r1, w["gamma"])
    Wg, Wu = np.concatenate(list(w["Wg"]), axis=0), np.concatenate(list(w["Wu"]), axis=0)
    Bd = np.concatenate(list(w["B"]), axis=1)
    g = x2 @ Wg.T
    r2 = r1 + ((g / (1.0 + np.exp(-g))) * (x2 @ Wu.T)) @ Bd.T
    for m in range(T):
        np.testing.assert_allclose(out["R1"][m], r1, atol=1e-11)
        np.testing.assert_allclose(out["R2"][m], r2, atol=1e-11)


def test_prefill_layer_p0_keeps_ranks_independent():
    """p = 0: no channel is shared, so rank m's output depends on rank m's residual stream only."""
    cfg, w = _tiny_prefill(p=0.0)
    kw = dict(batch=cfg.batch, seq=cfg.seq, heads_per_rank=cfg.n_heads // cfg.T, head_dim=cfg.head_dim, hs=0)
    a = O.prefill_layer_fwd(w["R"], w, **kw)
    R2 = w["R"].copy()
    R2[1] += 0.5
    b = O.prefill_layer_fwd(R2, w, **kw)
    assert np.array_equal(a["R2"][0], b["R2"][0])
    assert not np.array_equal(a["R2"][1], b["R2"][1])


# --------------------------------------------------------------------------- App. C closed forms
def test_comm_model_closed_forms():
    s, h = 2048, 4096
    assert O.comm_payload_elements(s, h, 1.0) == 2 * s * h
    for p in (0.75, 0.5, 0.25, 0.0):
        assert O.comm_payload_elements(s, h, p) / O.comm_payload_elements(s, h, 1.0) == p   # (1-p)*100% reduction
    # G counted from the layer's contractions (App. C: a 4h MLP, four h x h projections, QK^T and PV over s keys),
    # 2 FLOPs per multiply-add, divided over r devices -- not the closed form retyped
    gemms = [(s, h, h)] * 4 + [(s, 4 * h, h), (s, h, 4 * h), (s, s, h), (s, h, s)]        # (M, N, K)
    assert O.layer_flops_per_device(s, h, 8) == sum(2 * m * n * k for m, n, k in gemms) / 8
    # P(p) counted on the operator itself: the elements of one device's tensor that the partial channel-reduce sums
    # across ranks (those that differ from the rank's own input), two reduces per layer (attention and MLP outputs)
    for hh, p in ((16, 0.5), (16, 0.25), (24, 1.0), (8, 0.0)):
        ss, T = 6, 3
        Zt = _rng(77).standard_normal((T, ss, hh))
        Z = O.partial_channel_reduce(Zt, O.shared_channels(hh, p))
        assert 2 * int((Z[0] != Zt[0]).sum()) == O.comm_payload_elements(ss, hh, p)
    C, r = 3000.0, 8
    G = O.layer_flops_per_device(s, h, r)
    for p in (0.75, 0.5, 0.25, 0.0):
        t1 = G / C + O.comm_payload_elements(s, h, 1.0)
        tp = G / C + O.comm_payload_elements(s, h, p)
        assert abs((t1 - tp) / t1 - O.predicted_speedup(p, h, s, C, r)) < 1e-12


# --------------------------------------------------------------------------- input module sanity
def test_inputs_bf16_roundtrip_and_structure():
    x = np.array([1.0, -2.5, 3.140625, 1e-3, 65504.0], dtype=np.float32)
    b = I.f32_to_bf16_bits(x)
    np.testing.assert_array_equal(O.widen_bf16(b, np.float32), I.bf16_bits_to_f32(b))
    assert np.all(np.abs(I.bf16_bits_to_f32(b) - x) <= np.abs(x) * 2.0 ** -8)
    # ties round to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert I.f32_to_bf16_bits(np.array([1.0 + 2.0 ** -8], dtype=np.float32))[0] == 0x3F80
    assert I.f32_to_bf16_bits(np.array([1.0 + 3 * 2.0 ** -8], dtype=np.float32))[0] == 0x3F82
    d = make_inputs(I.C1, seed=0)
    assert d["X"].shape == (2, 256, 768) and d["A"].shape == (2, 1536, 768) and d["B"].shape == (2, 768, 1536)
    assert np.array_equal(d["R"][0, :, :384], d["R"][1, :, :384])
    assert not np.array_equal(d["R"][0, :, 384:], d["R"][1, :, 384:])
    d2 = make_inputs(I.C1, seed=0)
    assert all(np.array_equal(d[k], d2[k]) for k in d)
    assert abs(float(O.widen_bf16(d["A"]).std()) - 0.02) < 1e-3
