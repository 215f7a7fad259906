"""Seeded synthetic inputs for the partial-sync tensor-parallel block.

This module only draws random numbers and packs them as bf16 bit patterns
(numpy uint16).  It holds none of the method's arithmetic: no GEMM, no channel
reduce, no norm.  Both the CPU oracle (test infrastructure) and the HIP path are
fed the *same bits* produced here.

Shapes follow the paper's experimental models (130M-like h=768, 1.1B-like
h=2048, Llama2-7B h=4096 / ffn=11008 / 32 heads; TP 2/4/8; p in {1,.5,.25,0};
2K-token prompts), Sec. 5.  Real activations are replaced by N(0,1) draws and
weights by N(0, 0.02^2) draws because the cost of the block depends on shapes
only.

Draw order (one numpy Generator per call, PCG64, seeded): X, R, weights in the
order listed per kind (each rank-major), norm parameters, upstream gradients
dX', dR', then the KV cache.  Changing the order changes every stored value.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, Optional

import numpy as np

KIND_MLP_GELU = 0
KIND_MLP_SWIGLU = 1
KIND_ATTN = 2
KIND_DECODE = 3
KIND_PREFILL = 4
NORM_LAYERNORM = 0
NORM_RMSNORM = 1


@dataclasses.dataclass(frozen=True)
class BlockConfig:
    """Problem statement of one block: hidden h, TP degree T, sync fraction p, tokens."""

    name: str
    kind: int
    norm: int
    h: int
    T: int
    p: float
    batch: int
    seq: int
    ffn: int = 0
    n_heads: int = 0
    head_dim: int = 0
    kv_len: int = 0
    n_kv_heads: int = 0        # grouped-query attention: number of key / value heads (0 = n_heads, plain MHA)
    eps: float = 1e-5
    private_scale: float = 1.0
    rope_base: float = 10000.0

    @property
    def tokens(self) -> int:
        return self.batch * self.seq

    @property
    def f_r(self) -> int:
        return self.ffn // self.T

    @property
    def hd_r(self) -> int:
        """attention width owned by one rank = heads per rank * head_dim"""
        return (self.n_heads // self.T) * self.head_dim

    @property
    def kv_heads(self) -> int:
        return self.n_kv_heads if self.n_kv_heads > 0 else self.n_heads

    @property
    def kvd_r(self) -> int:
        """key (= value) width owned by one rank = kv heads per rank * head_dim"""
        return (self.kv_heads // self.T) * self.head_dim

    @property
    def qkv_r(self) -> int:
        """rows of one rank's fused projection shard: q heads, then k heads, then v heads"""
        return self.hd_r + 2 * self.kvd_r

    def with_(self, **kw) -> "BlockConfig":
        return dataclasses.replace(self, **kw)


# The five workload shapes of the benchmark definition.
C1 = BlockConfig("C1-gpt-mlp-tiny", KIND_MLP_GELU, NORM_LAYERNORM, h=768, T=2, p=0.5, batch=1, seq=256, ffn=3072)
C2 = BlockConfig("C2-gpt-mlp-1.1B", KIND_MLP_GELU, NORM_LAYERNORM, h=2048, T=4, p=0.5, batch=4, seq=2048, ffn=8192)
C3 = BlockConfig("C3-llama7b-mlp", KIND_MLP_SWIGLU, NORM_RMSNORM, h=4096, T=8, p=0.5, batch=2, seq=2048, ffn=11008)
C4 = BlockConfig("C4-llama7b-attn", KIND_ATTN, NORM_RMSNORM, h=4096, T=8, p=0.5, batch=1, seq=4096,
                 n_heads=32, head_dim=128)
C5 = BlockConfig("C5-llama7b-decode", KIND_DECODE, NORM_RMSNORM, h=4096, T=8, p=0.5, batch=64, seq=1,
                 ffn=11008, n_heads=32, head_dim=128, kv_len=2048)
# Beyond the five: one decoder layer over a whole prompt batch, the shape of the paper's time-to-first-token runs
# (Sec. 5.2: 2K-token prompts, batch 16 and up, Llama-7B dimensions, TP 8).
C6 = BlockConfig("C6-llama7b-prefill-layer", KIND_PREFILL, NORM_RMSNORM, h=4096, T=8, p=0.5, batch=16, seq=2048,
                 ffn=11008, n_heads=32, head_dim=128)
# The same layer with Llama-2-70B dimensions: grouped-query attention with 8 key / value heads, which caps the
# tensor-parallel degree at 8 (the paper's additional speed-up results).
C7 = BlockConfig("C7-llama70b-prefill-layer", KIND_PREFILL, NORM_RMSNORM, h=8192, T=8, p=0.5, batch=8, seq=2048,
                 ffn=28672, n_heads=64, head_dim=128, n_kv_heads=8)
CONFIGS = {c.name.split("-")[0]: c for c in (C1, C2, C3, C4, C5, C6, C7)}


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even), return the 16-bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float32 (format conversion only)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal_bf16(rng: np.random.Generator, shape, mean: float = 0.0, std: float = 1.0) -> np.ndarray:
    """Draw N(mean, std^2) in float32, chunked along axis 0 to bound memory, round to bf16 bits."""
    shape = tuple(int(s) for s in shape)
    out = np.empty(shape, dtype=np.uint16)
    flat = out.reshape(shape[0], -1) if len(shape) > 1 else out.reshape(1, -1)
    for i in range(flat.shape[0]):
        v = rng.standard_normal(flat.shape[1], dtype=np.float32)
        if std != 1.0:
            v *= np.float32(std)
        if mean != 0.0:
            v += np.float32(mean)
        flat[i] = f32_to_bf16_bits(v)
    return out


def _small_int_bf16(rng: np.random.Generator, shape, lo: int = -3, hi: int = 3) -> np.ndarray:
    """Small integers (exactly representable in bf16, sums of a few stay exact)."""
    return f32_to_bf16_bits(rng.integers(lo, hi + 1, size=shape).astype(np.float32))


def _activations(rng, cfg: BlockConfig, n: int, mode: str, hs_struct: Optional[int], with_x: bool = True):
    """X_m ~ N(0,1) per rank; R_m ~ N(0,1) with its shared columns equal on all ranks."""
    T, h = cfg.T, cfg.h
    X = _normal_bf16(rng, (T, n, h)) if with_x else None
    R = _normal_bf16(rng, (T, n, h))
    if mode == "replicated":
        if with_x:
            X[1:] = X[0]
        R[1:] = R[0]
    elif mode == "divergent":
        if hs_struct is None:
            raise ValueError("divergent inputs need hs_struct: how many leading residual columns are rank-equal")
        k = int(hs_struct)
        if k > 0:
            R[1:, :, :k] = R[0:1, :, :k]
    else:
        raise ValueError("mode must be 'divergent' or 'replicated'")
    return X, R


def make_inputs(cfg: BlockConfig, seed: int = 0, mode: str = "divergent", with_grads: bool = True,
                hs_struct: Optional[int] = None, weight_std: float = 0.02) -> Dict[str, np.ndarray]:
    """All tensors of one block call as bf16 bit patterns (uint16), keyed by name.

    mode='divergent': every rank has its own X_m (the method's normal operating
    point, Sec. 3.1); the residual's shared columns are copied from rank 0 and
    its private columns are independent.  mode='replicated': X_m = X_0 and
    R_m = R_0, the vanilla-TP special case used by the p=1 dense-equivalence check.
    hs_struct: how many leading residual columns are made rank-equal (required
    for mode='divergent').  It is a property of the data, chosen by the caller
    (tests pass the oracle's shared-channel count, the benchmark h/2 so that the
    same tensors serve every p); this module does not derive it from p.
    """
    rng = np.random.default_rng(seed)
    T, h, n = cfg.T, cfg.h, cfg.tokens
    d: Dict[str, np.ndarray] = {}
    if cfg.kind == KIND_PREFILL:       # the layer normalises R itself: no X is drawn
        _, d["R"] = _activations(rng, cfg, n, mode, hs_struct, with_x=False)
    else:
        d["X"], d["R"] = _activations(rng, cfg, n, mode, hs_struct)
    if cfg.kind == KIND_MLP_GELU:
        d["A"] = _normal_bf16(rng, (T, cfg.f_r, h), std=weight_std)        # column-parallel shard, [out,in]
        d["B"] = _normal_bf16(rng, (T, h, cfg.f_r), std=weight_std)        # row-parallel shard, [out,in]
    elif cfg.kind == KIND_MLP_SWIGLU:
        d["Wg"] = _normal_bf16(rng, (T, cfg.f_r, h), std=weight_std)
        d["Wu"] = _normal_bf16(rng, (T, cfg.f_r, h), std=weight_std)
        d["B"] = _normal_bf16(rng, (T, h, cfg.f_r), std=weight_std)
    elif cfg.kind == KIND_ATTN:
        d["Wqkv"] = _normal_bf16(rng, (T, cfg.qkv_r, h), std=weight_std)  # rows: q heads, k heads, v heads
        d["Wo"] = _normal_bf16(rng, (T, h, cfg.hd_r), std=weight_std)
    elif cfg.kind in (KIND_DECODE, KIND_PREFILL):
        d["gamma_attn"] = _normal_bf16(rng, (h,), mean=1.0, std=0.1)
        d["Wqkv"] = _normal_bf16(rng, (T, cfg.qkv_r, h), std=weight_std)
        d["Wo"] = _normal_bf16(rng, (T, h, cfg.hd_r), std=weight_std)
        d["Wg"] = _normal_bf16(rng, (T, cfg.f_r, h), std=weight_std)
        d["Wu"] = _normal_bf16(rng, (T, cfg.f_r, h), std=weight_std)
        d["B"] = _normal_bf16(rng, (T, h, cfg.f_r), std=weight_std)
    else:
        raise ValueError("unknown kind")
    d["gamma"] = _normal_bf16(rng, (h,), mean=1.0, std=0.1)
    if cfg.norm == NORM_LAYERNORM:
        d["beta"] = _normal_bf16(rng, (h,), std=0.1)
    if with_grads and cfg.kind not in (KIND_DECODE, KIND_PREFILL):
        d["dXo"] = _normal_bf16(rng, (T, n, h))   # dL/dX'
        d["dRo"] = _normal_bf16(rng, (T, n, h))   # dL/dR'
    if cfg.kind == KIND_DECODE:
        kvpr = cfg.kv_heads // cfg.T
        cap = cfg.kv_len + 1
        d["Kc"] = _normal_bf16(rng, (T, cfg.batch, kvpr, cap, cfg.head_dim))
        d["Vc"] = _normal_bf16(rng, (T, cfg.batch, kvpr, cap, cfg.head_dim))
    return d


def make_sync_inputs(T: int, n: int, h: int, seed: int = 0, integer: bool = False) -> Dict[str, np.ndarray]:
    """Partials Z~ [T,n,h] and residual R [T,n,h] for the stand-alone partial channel-reduce."""
    rng = np.random.default_rng(seed)
    if integer:
        return {"Zt": _small_int_bf16(rng, (T, n, h)), "R": _small_int_bf16(rng, (T, n, h))}
    return {"Zt": _normal_bf16(rng, (T, n, h)), "R": _normal_bf16(rng, (T, n, h))}


def make_norm_inputs(T: int, n: int, h: int, layernorm: bool, seed: int = 0) -> Dict[str, np.ndarray]:
    rng = np.random.default_rng(seed)
    d = {"R": _normal_bf16(rng, (T, n, h), mean=0.25, std=1.5),
         "gamma": _normal_bf16(rng, (h,), mean=1.0, std=0.1)}
    if layernorm:
        d["beta"] = _normal_bf16(rng, (h,), std=0.1)
    d["dXo"] = _normal_bf16(rng, (T, n, h))
    d["dRo"] = _normal_bf16(rng, (T, n, h))
    return d


def make_gemm_inputs(G: int, M: int, N: int, K: int, seed: int = 0, std_a: float = 1.0,
                     std_b: float = 0.02) -> Dict[str, np.ndarray]:
    """Operands of a grouped GEMM C_g[M,N] = sum_k a_g[M,K] b_g[N,K] (both K-contiguous)."""
    rng = np.random.default_rng(seed)
    return {"a": _normal_bf16(rng, (G, M, K), std=std_a), "b": _normal_bf16(rng, (G, N, K), std=std_b)}
