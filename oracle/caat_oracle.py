"""CPU oracle for the partial-sync tensor-parallel block (CAAT-Net).

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module;
only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg call it.
It shares no code with the HIP library and never calls it.

Everything here is the plain definition from the paper, written with numpy in
float64 (pass dtype=np.float32 for the fp32 variant): the method is exact -- a
re-association of sums plus a channel mask -- so the oracle is the definition
written out, with numpy's matmul / scipy's erf as library steps and no tiling,
fusion or reordering.  Tensors carry an explicit leading rank index m, as in
the paper's index notation of App. A.2 (X_{ijm}, Z_{ilm}).

Layouts (row-major): activations [T, n, h]; column-parallel shard A_m stored
[f/T, h] (out, in); row-parallel shard B_m stored [h, f/T] (out, in); QKV shard
[3*hd_r, h] with rows q|k|v, heads contiguous (grouped-query attention: fewer k and v rows); O shard [h, hd_r].

Pins (tests/test_oracle_*.py): every function below is checked against a
closed form, an invariant, brute-force Python loops on tiny shapes or central
finite differences.  One statement is "parity unpinned": that fp32 rather than
16-bit accumulation of the backward reduce is needed for training to converge
(Sec. 4, App. E.1) is a training outcome; only the arithmetic rule is checked.
"""
from __future__ import annotations

import math
from typing import Dict, Optional

import numpy as np
from scipy.special import erf as _erf

LAYERNORM = 0
RMSNORM = 1


# ----------------------------------------------------------------------------- formats
def widen_bf16(bits: np.ndarray, dtype=np.float64) -> np.ndarray:
    """bf16 bit pattern -> real number, exactly (bf16 is the top half of an IEEE float32)."""
    u = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(dtype)


# ----------------------------------------------------------------------------- Sec. 3, Eq. A3
def shared_channels(h: int, p: float) -> int:
    """Number of shared channels: the first floor(h*p) channels (Sec. 3; case split of Eq. A3)."""
    if not (0.0 <= p <= 1.0):
        raise ValueError("p must lie in [0,1]")
    return int(math.floor(h * p))


def partial_channel_reduce(Zt: np.ndarray, hs: int, private_scale: float = 1.0) -> np.ndarray:
    """Eq. A3 / A5, second line: Z_{ilm} = sum_m' Zt_{ilm'} if l < hs, else Zt_{ilm}.

    Zt: [T, n, h] per-rank partial outputs.  Private channels are multiplied by
    private_scale (Sec. 4 'Private channel scaling'; 1.0 switches it off).
    """
    T, n, h = Zt.shape
    if not (0 <= hs <= h):
        raise ValueError("hs out of range")
    Z = np.empty_like(Zt)
    total = np.zeros((n, hs), dtype=Zt.dtype)
    for m in range(T):                      # ascending rank order
        total = total + Zt[m, :, :hs]
    for m in range(T):
        Z[m, :, :hs] = total                # shared channels: same value on every rank
        Z[m, :, hs:] = private_scale * Zt[m, :, hs:]   # private channels stay rank-local
    return Z


# ----------------------------------------------------------------------------- activations
def gelu(x):
    """x * Phi(x), Phi the standard normal CDF (exact erf form)."""
    return 0.5 * x * (1.0 + _erf(x / math.sqrt(2.0)))


def gelu_grad(x):
    """d/dx [x Phi(x)] = Phi(x) + x phi(x)."""
    return 0.5 * (1.0 + _erf(x / math.sqrt(2.0))) + x * np.exp(-0.5 * x * x) / math.sqrt(2.0 * math.pi)


def sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


def silu(x):
    return x * sigmoid(x)


def silu_grad(x):
    s = sigmoid(x)
    return s * (1.0 + x * (1.0 - s))


# ----------------------------------------------------------------------------- Norm (Sec. 4, X_m = Norm(.))
def norm_fwd(Rp: np.ndarray, gamma: np.ndarray, beta: Optional[np.ndarray], kind: int, eps: float):
    """Per rank, per token normalisation over the hidden axis.

    LayerNorm: (x - mean) / sqrt(var + eps) * gamma + beta, biased variance.
    RMSNorm:   x / sqrt(mean(x^2) + eps) * gamma.
    Returns (X', xhat, rstd).
    """
    if kind == LAYERNORM:
        mu = Rp.mean(axis=-1, keepdims=True)
        xc = Rp - mu
        var = (xc * xc).mean(axis=-1, keepdims=True)
        rstd = 1.0 / np.sqrt(var + eps)
        xhat = xc * rstd
        out = xhat * gamma + (beta if beta is not None else 0.0)
    elif kind == RMSNORM:
        ms = (Rp * Rp).mean(axis=-1, keepdims=True)
        rstd = 1.0 / np.sqrt(ms + eps)
        xhat = Rp * rstd
        out = xhat * gamma
    else:
        raise ValueError("unknown norm")
    return out, xhat, rstd


def norm_bwd(dXo: np.ndarray, Rp: np.ndarray, gamma: np.ndarray, kind: int, eps: float):
    """Gradient of norm_fwd w.r.t. its input and parameters.

    Returns (dRp_from_norm [T,n,h], dgamma_m [T,h], dbeta_m [T,h]): parameter
    gradients are still per rank here; they are summed over ranks by the caller
    (Sec. 4: norm parameters must be synchronised before the weight update).
    """
    _, xhat, rstd = norm_fwd(Rp, gamma, None, kind, eps)
    dxhat = dXo * gamma
    if kind == LAYERNORM:
        dx = rstd * (dxhat - dxhat.mean(axis=-1, keepdims=True)
                     - xhat * (dxhat * xhat).mean(axis=-1, keepdims=True))
    else:
        dx = rstd * (dxhat - xhat * (dxhat * xhat).mean(axis=-1, keepdims=True))
    dgamma_m = (dXo * xhat).sum(axis=1)
    dbeta_m = dXo.sum(axis=1)
    return dx, dgamma_m, dbeta_m


# ----------------------------------------------------------------------------- MLP block, Eq. 6-8 / A3
def mlp_block_fwd(X, R, W: Dict[str, np.ndarray], gamma, beta, *, swiglu: bool, norm: int, hs: int,
                  eps: float = 1e-5, private_scale: float = 1.0) -> Dict[str, np.ndarray]:
    """Forward of one MLP sub-block with partial channel-reduce, then residual and norm.

    X, R: [T, n, h] real arrays (already widened).  W: 'A','B' (GELU) or
    'Wg','Wu','B' (SwiGLU), shapes as in the module docstring.
      P_m  = X_m A_m            (column-parallel, Eq. A3 inner sum)
      Y_m  = sigma(P_m)         or silu(X_m Wg_m) * (X_m Wu_m)
      Zt_m = Y_m B_m            (row-parallel partial sum)
      Z    = PCR_p(Zt)          (Eq. A3 case split)
      R'_m = R_m + Z_m ; X'_m = Norm(R'_m)
    """
    T = X.shape[0]
    out: Dict[str, np.ndarray] = {}
    Ys, Zts, Ps, Pus = [], [], [], []
    for m in range(T):
        if swiglu:
            Pg = X[m] @ W["Wg"][m].T
            Pu = X[m] @ W["Wu"][m].T
            Y = silu(Pg) * Pu
            Ps.append(Pg)
            Pus.append(Pu)
        else:
            P = X[m] @ W["A"][m].T
            Y = gelu(P)
            Ps.append(P)
        Ys.append(Y)
        Zts.append(Y @ W["B"][m].T)
    out["P"] = np.stack(Ps)
    if swiglu:
        out["Pu"] = np.stack(Pus)
    out["Y"] = np.stack(Ys)
    out["Zt"] = np.stack(Zts)
    out["Z"] = partial_channel_reduce(out["Zt"], hs, private_scale)
    out["Rp"] = R + out["Z"]
    out["Xp"], _, _ = norm_fwd(out["Rp"], gamma, beta, norm, eps)
    return out


def mlp_block_bwd(X, fwd: Dict[str, np.ndarray], W: Dict[str, np.ndarray], gamma, dXo, dRo, *, swiglu: bool,
                  norm: int, hs: int, eps: float = 1e-5, private_scale: float = 1.0) -> Dict[str, np.ndarray]:
    """Backward of mlp_block_fwd given dL/dX' (dXo) and dL/dR' (dRo), both [T,n,h].

    The reduce sits where the forward one sits (Fig. 2b): first back-propagate
    through the norm per rank, G_m = dRo_m + NormBwd(dXo_m); the residual branch
    takes dR_m = G_m un-reduced (App. B); the same partial channel-reduce is then
    applied to G (it is linear and its own adjoint); the GEMM chain rule follows
    per rank with NO reduce at the column-parallel input.  Norm-parameter
    gradients are summed over ranks.
    """
    T = X.shape[0]
    dn, dgamma_m, dbeta_m = norm_bwd(dXo, fwd["Rp"], gamma, norm, eps)
    G = dRo + dn
    dZt = partial_channel_reduce(G, hs, private_scale)
    g: Dict[str, np.ndarray] = {"dR": G, "dZt": dZt, "dgamma": dgamma_m.sum(axis=0)}
    if norm == LAYERNORM:
        g["dbeta"] = dbeta_m.sum(axis=0)
    dXs, dBs, dAs, dWgs, dWus, dPs, dPus = [], [], [], [], [], [], []
    for m in range(T):
        dY = dZt[m] @ W["B"][m]               # [n,h] x [h,f_r]
        dBs.append(dZt[m].T @ fwd["Y"][m])    # [h,f_r]
        if swiglu:
            Pg, Pu = fwd["P"][m], fwd["Pu"][m]
            dPg = dY * Pu * silu_grad(Pg)
            dPu = dY * silu(Pg)
            dWgs.append(dPg.T @ X[m])
            dWus.append(dPu.T @ X[m])
            dXs.append(dPg @ W["Wg"][m] + dPu @ W["Wu"][m])
            dPs.append(dPg)
            dPus.append(dPu)
        else:
            dP = dY * gelu_grad(fwd["P"][m])
            dAs.append(dP.T @ X[m])
            dXs.append(dP @ W["A"][m])
            dPs.append(dP)
    g["dX"] = np.stack(dXs)
    g["dB"] = np.stack(dBs)
    g["dP"] = np.stack(dPs)
    if swiglu:
        g["dWg"] = np.stack(dWgs)
        g["dWu"] = np.stack(dWus)
        g["dPu"] = np.stack(dPus)
    else:
        g["dA"] = np.stack(dAs)
    return g


# ----------------------------------------------------------------------------- attention, Eq. A5
def rope(x: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotary position embedding on the last axis d of x[..., s, d] for positions pos[s].

    Pairs (j, j + d/2), angle pos * base^(-2j/d):
      x'[j]       = x[j] cos - x[j+d/2] sin
      x'[j+d/2]   = x[j+d/2] cos + x[j] sin
    (Not in the paper; fixed by the workload definition.)
    """
    d = x.shape[-1]
    half = d // 2
    j = np.arange(half, dtype=np.float64)
    inv = base ** (-2.0 * j / d)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv[None, :]
    c, s = np.cos(ang).astype(x.dtype), np.sin(ang).astype(x.dtype)
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def causal_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, q_pos0: int = 0) -> np.ndarray:
    """softmax(q k^T / sqrt(d) + causal mask) v for one head.

    q: [sq, d], k, v: [sk, d].  Query i sits at absolute position q_pos0 + i and
    sees keys 0 .. q_pos0 + i.
    """
    sq, d = q.shape
    sk = k.shape[0]
    s = (q @ k.T) / math.sqrt(d)
    qi = np.arange(sq)[:, None] + q_pos0
    kj = np.arange(sk)[None, :]
    s = np.where(kj <= qi, s, -np.inf)
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    return (e / e.sum(axis=-1, keepdims=True)) @ v


def attn_block_fwd(X, R, Wqkv, Wo, gamma, beta, *, batch: int, seq: int, heads_per_rank: int, head_dim: int,
                   norm: int, hs: int, eps: float = 1e-5, private_scale: float = 1.0,
                   rope_base: float = 10000.0, kv_heads_per_rank: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Attention sub-block with partial channel-reduce (Eq. A5), then residual and norm.

    Per rank m: q,k,v = X_m Wq_m, X_m Wk_m, X_m Wv_m; RoPE on q,k; causal
    attention per head within each sequence; Zt_m = H_m O_m; Z = PCR(Zt);
    R' = R + Z; X' = Norm(R').  X, R: [T, batch*seq, h].
    Grouped-query attention (the 34B / 70B models of App. E, additional speed-up results): a rank owns kv_heads_per_rank key / value heads
    (default: one per query head); query head a reads key / value head a // (heads_per_rank / kv_heads_per_rank).
    The projection shard has heads_per_rank*d q rows, then kv_heads_per_rank*d k rows, then as many v rows.
    """
    T, n, h = X.shape
    d = head_dim
    hd = heads_per_rank * d
    kvpr = heads_per_rank if kv_heads_per_rank is None else kv_heads_per_rank
    grp = heads_per_rank // kvpr
    kvd = kvpr * d
    pos = np.arange(seq)
    Hs, Zts, Qs, Ks, Vs = [], [], [], [], []
    for m in range(T):
        qkv = X[m] @ Wqkv[m].T                       # [n, hd + 2*kvd]
        H = np.empty((n, hd), dtype=X.dtype)
        Qm = np.empty((batch, heads_per_rank, seq, d), dtype=X.dtype)
        Km = np.empty((batch, kvpr, seq, d), dtype=X.dtype)
        Vm = np.empty_like(Km)
        for b in range(batch):
            rows = slice(b * seq, (b + 1) * seq)
            for c in range(kvpr):
                Km[b, c] = rope(qkv[rows, hd + c * d:hd + (c + 1) * d], pos, rope_base)
                Vm[b, c] = qkv[rows, hd + kvd + c * d:hd + kvd + (c + 1) * d]
            for a in range(heads_per_rank):
                q = rope(qkv[rows, a * d:(a + 1) * d], pos, rope_base)
                Qm[b, a] = q
                H[rows, a * d:(a + 1) * d] = causal_attention(q, Km[b, a // grp], Vm[b, a // grp])
        Hs.append(H)
        Qs.append(Qm)
        Ks.append(Km)
        Vs.append(Vm)
        Zts.append(H @ Wo[m].T)
    out = {"H": np.stack(Hs), "Zt": np.stack(Zts), "Q": np.stack(Qs), "K": np.stack(Ks), "V": np.stack(Vs)}
    out["Z"] = partial_channel_reduce(out["Zt"], hs, private_scale)
    out["Rp"] = R + out["Z"]
    out["Xp"], _, _ = norm_fwd(out["Rp"], gamma, beta, norm, eps)
    return out


def rope_adjoint(dy: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Gradient of rope w.r.t. its input: rope is, per pair (j, j+d/2), a plane rotation by +angle, so its
    transpose (= adjoint, the Jacobian is orthogonal) is the rotation by -angle:
      dx[j]     =  dy[j] cos + dy[j+d/2] sin
      dx[j+d/2] = -dy[j] sin + dy[j+d/2] cos
    """
    d = dy.shape[-1]
    half = d // 2
    j = np.arange(half, dtype=np.float64)
    inv = base ** (-2.0 * j / d)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv[None, :]
    c, s = np.cos(ang).astype(dy.dtype), np.sin(ang).astype(dy.dtype)
    g1, g2 = dy[..., :half], dy[..., half:]
    return np.concatenate([g1 * c + g2 * s, g2 * c - g1 * s], axis=-1)


def causal_attention_bwd(q: np.ndarray, k: np.ndarray, v: np.ndarray, dO: np.ndarray, q_pos0: int = 0):
    """Gradient of causal_attention for one head, chain rule written out.

    With S = q k^T / sqrt(d) (masked), P = softmax_rows(S), O = P v:
      dv = P^T dO;  dP = dO v^T;  dS_ij = P_ij (dP_ij - sum_j' dP_ij' P_ij')  (softmax Jacobian);
      dq = dS k / sqrt(d);  dk = dS^T q / sqrt(d).   Masked entries have P = 0, hence dS = 0.
    Returns (dq, dk, dv).
    """
    sq, d = q.shape
    sk = k.shape[0]
    s = (q @ k.T) / math.sqrt(d)
    qi = np.arange(sq)[:, None] + q_pos0
    kj = np.arange(sk)[None, :]
    s = np.where(kj <= qi, s, -np.inf)
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    P = e / e.sum(axis=-1, keepdims=True)
    dv = P.T @ dO
    dP = dO @ v.T
    dS = P * (dP - (dP * P).sum(axis=-1, keepdims=True))
    dq = (dS @ k) / math.sqrt(d)
    dk = (dS.T @ q) / math.sqrt(d)
    return dq, dk, dv


def attn_block_bwd(X, fwd: Dict[str, np.ndarray], Wqkv, Wo, gamma, dXo, dRo, *, batch: int, seq: int,
                   heads_per_rank: int, head_dim: int, norm: int, hs: int, eps: float = 1e-5,
                   private_scale: float = 1.0, rope_base: float = 10000.0,
                   kv_heads_per_rank: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Backward of attn_block_fwd given dL/dX' (dXo) and dL/dR' (dRo), both [T,n,h].

    Same placement as the MLP block (Fig. 2b, Sec. 4): norm backward per rank first, G_m = dRo_m + NormBwd(dXo_m),
    dR_m = G_m un-reduced (App. B), the partial channel-reduce on G, then the chain rule of Eq. A5 per rank:
      dH_m = dZt_m O_m ; dO_m = dZt_m^T H_m ; per (sequence, head) the attention gradient, the RoPE adjoint on
      dq, dk ; dqkv_m = [dq | dk | dv] ; dX_m = dqkv_m Wqkv_m (no reduce over ranks) ; dWqkv_m = dqkv_m^T X_m.
    fwd is attn_block_fwd's result (needs Rp, H and the rotated Q, K and V).  With grouped-query attention a
    key / value head collects the gradients of every query head that read it.
    """
    T, n, h = X.shape
    d = head_dim
    hd = heads_per_rank * d
    kvpr = heads_per_rank if kv_heads_per_rank is None else kv_heads_per_rank
    grp = heads_per_rank // kvpr
    kvd = kvpr * d
    pos = np.arange(seq)
    dn, dgamma_m, dbeta_m = norm_bwd(dXo, fwd["Rp"], gamma, norm, eps)
    G = dRo + dn
    dZt = partial_channel_reduce(G, hs, private_scale)
    g: Dict[str, np.ndarray] = {"dR": G, "dZt": dZt, "dgamma": dgamma_m.sum(axis=0)}
    if norm == LAYERNORM:
        g["dbeta"] = dbeta_m.sum(axis=0)
    dXs, dWos, dWqkvs, dHs, dqkvs = [], [], [], [], []
    for m in range(T):
        dH = dZt[m] @ Wo[m]                       # [n,h] x [h,hd]
        dWos.append(dZt[m].T @ fwd["H"][m])       # [h,hd]
        dqkv = np.empty((n, hd + 2 * kvd), dtype=X.dtype)
        for b in range(batch):
            rows = slice(b * seq, (b + 1) * seq)
            for c in range(kvpr):
                dk_sum = np.zeros((seq, d), dtype=X.dtype)
                dv_sum = np.zeros((seq, d), dtype=X.dtype)
                for a in range(c * grp, (c + 1) * grp):      # the query heads that read key / value head c
                    cols = slice(a * d, (a + 1) * d)
                    dq, dk, dv = causal_attention_bwd(fwd["Q"][m, b, a], fwd["K"][m, b, c], fwd["V"][m, b, c],
                                                      dH[rows, cols])
                    dqkv[rows, a * d:(a + 1) * d] = rope_adjoint(dq, pos, rope_base)
                    dk_sum = dk_sum + dk
                    dv_sum = dv_sum + dv
                dqkv[rows, hd + c * d:hd + (c + 1) * d] = rope_adjoint(dk_sum, pos, rope_base)
                dqkv[rows, hd + kvd + c * d:hd + kvd + (c + 1) * d] = dv_sum
        dHs.append(dH)
        dqkvs.append(dqkv)
        dXs.append(dqkv @ Wqkv[m])                # [n,hd+2kvd] x [hd+2kvd,h]
        dWqkvs.append(dqkv.T @ X[m])              # [hd+2kvd,h]
    g["dH"] = np.stack(dHs)
    g["dqkv"] = np.stack(dqkvs)
    g["dX"] = np.stack(dXs)
    g["dWo"] = np.stack(dWos)
    g["dWqkv"] = np.stack(dWqkvs)
    return g


def decode_layer_fwd(R, W: Dict[str, np.ndarray], Kc, Vc, *, kv_len: int, heads_per_rank: int, head_dim: int,
                     hs: int, eps: float = 1e-5, private_scale: float = 1.0, rope_base: float = 10000.0,
                     kv_heads_per_rank: Optional[int] = None) -> Dict[str, np.ndarray]:
    """One Llama-style decoder layer for one new token per sequence (RMSNorm, SwiGLU).

    R: [T, b, h] per-rank residual stream.  Kc, Vc: [T, b, kv_heads_per_rank, cap, d]
    caches whose first kv_len positions are filled (keys already rotated); the
    new token sits at position kv_len and its k, v are appended at that index.
      X1 = RMSNorm(R; gamma_attn); q,k,v = X1 Wqkv; RoPE(q,k at kv_len)
      H  = softmax(q K^T / sqrt(d)) V over kv_len+1 keys;  Zt = H Wo
      R1 = R + PCR(Zt);  X2 = RMSNorm(R1; gamma)
      Zt2 = (silu(X2 Wg) * (X2 Wu)) B;  R2 = R1 + PCR(Zt2)
    Returns R1, R2, the appended k, v rows and intermediates.
    """
    T, b, h = R.shape
    d = head_dim
    hd = heads_per_rank * d
    kvpr = heads_per_rank if kv_heads_per_rank is None else kv_heads_per_rank
    grp = heads_per_rank // kvpr
    kvd = kvpr * d
    X1, _, _ = norm_fwd(R, W["gamma_attn"], None, RMSNORM, eps)
    Zt = np.empty_like(R)
    k_new = np.empty((T, b, kvpr, d), dtype=R.dtype)
    v_new = np.empty_like(k_new)
    Hall = np.empty((T, b, hd), dtype=R.dtype)
    pos = np.array([kv_len])
    for m in range(T):
        qkv = X1[m] @ W["Wqkv"][m].T
        for s in range(b):
            for c in range(kvpr):
                k = rope(qkv[s:s + 1, hd + c * d:hd + (c + 1) * d], pos, rope_base)
                v = qkv[s:s + 1, hd + kvd + c * d:hd + kvd + (c + 1) * d]
                k_new[m, s, c], v_new[m, s, c] = k[0], v[0]
                Kall = np.concatenate([Kc[m, s, c, :kv_len], k], axis=0)
                Vall = np.concatenate([Vc[m, s, c, :kv_len], v], axis=0)
                for a in range(c * grp, (c + 1) * grp):
                    q = rope(qkv[s:s + 1, a * d:(a + 1) * d], pos, rope_base)
                    Hall[m, s, a * d:(a + 1) * d] = causal_attention(q, Kall, Vall, q_pos0=kv_len)[0]
        Zt[m] = Hall[m] @ W["Wo"][m].T
    R1 = R + partial_channel_reduce(Zt, hs, private_scale)
    X2, _, _ = norm_fwd(R1, W["gamma"], None, RMSNORM, eps)
    Zt2 = np.empty_like(R)
    for m in range(T):
        Y = silu(X2[m] @ W["Wg"][m].T) * (X2[m] @ W["Wu"][m].T)
        Zt2[m] = Y @ W["B"][m].T
    R2 = R1 + partial_channel_reduce(Zt2, hs, private_scale)
    return {"X1": X1, "H": Hall, "Zt": Zt, "R1": R1, "X2": X2, "Zt2": Zt2, "R2": R2, "k_new": k_new, "v_new": v_new}


def prefill_layer_fwd(R, W: Dict[str, np.ndarray], *, batch: int, seq: int, heads_per_rank: int, head_dim: int,
                      hs: int, eps: float = 1e-5, private_scale: float = 1.0, rope_base: float = 10000.0,
                      kv_heads_per_rank: Optional[int] = None) -> Dict[str, np.ndarray]:
    """One Llama-style decoder layer over a whole prompt (the time-to-first-token workload of Sec. 5.2): the
    attention sub-block of Eq. A5 followed by the SwiGLU MLP sub-block of Eq. A3, each closed by its partial
    channel-reduce and residual add, RMSNorm in front of each (Sec. 4).

    R: [T, batch*seq, h] per-rank residual stream.  W as for decode_layer_fwd.
      X1 = RMSNorm(R; gamma_attn); attention sub-block on (X1, R) -> R1 = R + PCR(H Wo), X2 = RMSNorm(R1; gamma)
      MLP sub-block on (X2, R1)  -> R2 = R1 + PCR((silu(X2 Wg) * (X2 Wu)) B)
    Returns R1, X2, R2, intermediates and the rotated keys K and the values V [T, batch, kv_heads_per_rank, seq, d]
    that a KV cache holds after the prompt.
    """
    X1, _, _ = norm_fwd(R, W["gamma_attn"], None, RMSNORM, eps)
    att = attn_block_fwd(X1, R, W["Wqkv"], W["Wo"], W["gamma"], None, batch=batch, seq=seq,
                         heads_per_rank=heads_per_rank, head_dim=head_dim, norm=RMSNORM, hs=hs, eps=eps,
                         private_scale=private_scale, rope_base=rope_base, kv_heads_per_rank=kv_heads_per_rank)
    R1, X2 = att["Rp"], att["Xp"]
    T = R.shape[0]
    Zt2 = np.empty_like(R)
    Ys = []
    for m in range(T):
        Y = silu(X2[m] @ W["Wg"][m].T) * (X2[m] @ W["Wu"][m].T)
        Ys.append(Y)
        Zt2[m] = Y @ W["B"][m].T
    R2 = R1 + partial_channel_reduce(Zt2, hs, private_scale)
    return {"X1": X1, "Q": att["Q"], "K": att["K"], "V": att["V"], "H": att["H"], "Zt": att["Zt"], "R1": R1, "X2": X2,
            "Y": np.stack(Ys), "Zt2": Zt2, "R2": R2}


# ----------------------------------------------------------------------------- App. C closed forms
def comm_payload_elements(s: int, h: int, p: float) -> float:
    """P(p) = 2 s h p elements per device per layer forward (App. C)."""
    return 2.0 * s * h * p


def layer_flops_per_device(s: int, h: int, r: int) -> float:
    """G = (24 s h^2 + 4 s^2 h) / r (App. C)."""
    return (24.0 * s * h * h + 4.0 * s * s * h) / r


def predicted_speedup(p: float, h: int, s: int, C: float, r: int) -> float:
    """(T(1) - T(p)) / T(1) = (1 - p) / (1 + (12 h + 2 s) / (C r)), with T(p) = G/C + P(p)."""
    return (1.0 - p) / (1.0 + (12.0 * h + 2.0 * s) / (C * r))
