"""GPU parity of the prefill decoder layer (a whole prompt through attention + SwiGLU MLP, each with its partial
channel-reduce, KV cache filled) against the CPU oracle, through the C ABI; and the prefill -> decode hand-over."""
import numpy as np
import pytest

from oracle import caat_oracle as O
from paper_2506_19645_amd import binding as B
from paper_2506_19645_amd import inputs as I
from tests.util import assert_close, bits_to_f64, make_inputs, hs_of

pytestmark = pytest.mark.gpu


def layer_weights(d):
    return [B.to_device(d["gamma_attn"]), B.to_device(d["Wqkv"]), B.to_device(d["Wo"]), B.to_device(d["gamma"]),
            B.to_device(np.concatenate([d["Wg"], d["Wu"]], axis=1)), B.to_device(d["B"])]


def run_prefill(cfg, d, kv_cap=None, keep=("X1", "H", "R1", "X2"), reduce_in_gemm=False, separate_reduce=False):
    import torch
    desc = B.make_desc(cfg, kv_cap=kv_cap, reduce_in_gemm=reduce_in_gemm, separate_reduce=separate_reduce)
    T, n, h, hd, hpr = cfg.T, cfg.tokens, cfg.h, cfg.hd_r, cfg.kv_heads // cfg.T     # hpr: key / value heads per rank
    weights = layer_weights(d)
    r = B.to_device(d["R"])
    cap = desc.kv_cap
    kc = torch.zeros((T, cfg.batch, hpr, cap, cfg.head_dim), dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    r_out = torch.empty_like(r)
    ws = torch.zeros(B.workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    B.block_fwd(desc, weights, None, r, r_out, None, ws, kv_k=kc, kv_v=vc)
    torch.cuda.synchronize()
    L = B.workspace_layout(desc)

    def ws_bits(off, nbytes, shape):
        return ws[off:off + nbytes].view(torch.int16).cpu().numpy().view(np.uint16).reshape(shape)

    shapes = {"X1": (L.off_X1, L.bytes_X1, (T, n, h)), "H": (L.off_H, L.bytes_H, (T, n, hd)),
              "R1": (L.off_R1, L.bytes_R1, (T, n, h)), "X2": (L.off_X2, L.bytes_X2, (T, n, h))}
    out = {"R2_bits": B.to_host_bits(r_out), "Kc_bits": B.to_host_bits(kc), "Vc_bits": B.to_host_bits(vc),
           "kc_dev": kc, "vc_dev": vc, "weights_dev": weights}
    for name in keep:
        out[name + "_bits"] = ws_bits(*shapes[name])
    return out


def oracle_prefill(cfg, d):
    w = {k: O.widen_bf16(v) for k, v in d.items()}
    return w, O.prefill_layer_fwd(w["R"], w, batch=cfg.batch, seq=cfg.seq, heads_per_rank=cfg.n_heads // cfg.T,
                                  head_dim=cfg.head_dim, hs=hs_of(cfg), eps=cfg.eps, private_scale=cfg.private_scale,
                                  rope_base=cfg.rope_base, kv_heads_per_rank=cfg.kv_heads // cfg.T)


def check_prefill(cfg, d, got, ref, rows=None):
    """rows: token rows of `got` that `ref` covers (None = all)."""
    sel = (lambda a: a) if rows is None else (lambda a: a[:, rows])
    for name in ("X1", "H", "R1", "X2"):
        if name + "_bits" in got:
            assert_close(bits_to_f64(sel(got[name + "_bits"])), ref[name], name)
    assert_close(bits_to_f64(sel(got["R2_bits"])), ref["R2"], "R2")


def _cfg(T, batch, seq, heads, ffn, p, scale=1.0, kv_heads=0):
    return I.BlockConfig("pre", I.KIND_PREFILL, I.NORM_RMSNORM, h=heads * 128, T=T, p=p, batch=batch, seq=seq, ffn=ffn,
                         n_heads=heads, head_dim=128, private_scale=scale, n_kv_heads=kv_heads)


@pytest.mark.parametrize("T,batch,seq,heads,ffn,p,scale,kv_heads", [
    (2, 1, 64, 2, 2 * 256, 0.5, 1.0, 0),         # one key block
    (2, 3, 200, 4, 2 * 344, 0.5, 1.0, 0),        # three ragged sequences, ragged ffn shard
    (4, 2, 130, 4, 4 * 128, 0.25, 2.0, 0),       # private-channel scaling sqrt(T)
    (1, 1, 333, 2, 512, 1.0, 1.0, 0),            # T = 1
    (2, 2, 70, 2, 2 * 256, 0.0, 1.0, 0),         # p = 0
    (2, 2, 200, 8, 2 * 256, 0.5, 1.0, 2),        # grouped-query attention
    (16, 1, 100, 32, 16 * 128, 0.5, 1.0, 0),     # tensor-parallel degree 16 (Sec. 5's largest): 32 heads, 2 per rank
    (16, 2, 70, 32, 16 * 136, 0.25, 4.0, 16),    # T = 16 with grouped-query attention (one key / value head per rank), sqrt(T)
])
def test_prefill_layer(T, batch, seq, heads, ffn, p, scale, kv_heads):
    cfg = _cfg(T, batch, seq, heads, ffn, p, scale, kv_heads)
    d = make_inputs(cfg, seed=41, weight_std=0.05 if cfg.h < 4096 else 0.02)   # h = 4096: scores stay O(1), as in the benchmark
    got = run_prefill(cfg, d, kv_cap=seq + 3)
    w, ref = oracle_prefill(cfg, d)
    check_prefill(cfg, d, got, ref)
    # the cache holds the prompt's rotated keys and values at positions 0..seq-1 and nothing else was written
    assert_close(bits_to_f64(got["Kc_bits"][:, :, :, :seq]), ref["K"], "K cache")
    assert_close(bits_to_f64(got["Vc_bits"][:, :, :, :seq]), ref["V"], "V cache")
    assert not got["Kc_bits"][:, :, :, seq:].any() and not got["Vc_bits"][:, :, :, seq:].any()
    hs = hs_of(cfg)
    if hs > 0 and T > 1:
        for m in range(1, T):
            assert np.array_equal(got["R2_bits"][m, :, :hs], got["R2_bits"][0, :, :hs])


def test_prefill_then_decode_matches_longer_prefill():
    """Prefill L tokens on the GPU, then decode token L over the cache the prefill left: the result must match the
    oracle's prefill over L+1 tokens in its last row (and the cache row L must hold that token's key and value)."""
    import torch
    T, b, heads, ffn, L = 2, 3, 4, 2 * 256, 150
    full = _cfg(T, b, L + 1, heads, ffn, 0.5)
    d = make_inputs(full, seed=42, weight_std=0.05)
    w, ref = oracle_prefill(full, d)
    R = d["R"].reshape(T, b, L + 1, full.h)
    pre_cfg = _cfg(T, b, L, heads, ffn, 0.5)
    d_pre = dict(d, R=np.ascontiguousarray(R[:, :, :L]).reshape(T, b * L, full.h))
    got = run_prefill(pre_cfg, d_pre, kv_cap=L + 1, keep=())
    dec_cfg = I.BlockConfig("dec", I.KIND_DECODE, I.NORM_RMSNORM, h=full.h, T=T, p=0.5, batch=b, seq=1, ffn=ffn,
                            n_heads=heads, head_dim=128, kv_len=L)
    desc = B.make_desc(dec_cfg)
    r = B.to_device(np.ascontiguousarray(R[:, :, L]))
    r_out = torch.empty_like(r)
    ws = torch.zeros(B.workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    B.block_fwd(desc, got["weights_dev"], None, r, r_out, None, ws, kv_k=got["kc_dev"], kv_v=got["vc_dev"])
    torch.cuda.synchronize()
    last = [s * (L + 1) + L for s in range(b)]
    assert_close(bits_to_f64(B.to_host_bits(r_out)), ref["R2"][:, last], "R2 of the decoded token")
    kc = bits_to_f64(B.to_host_bits(got["kc_dev"]))
    vc = bits_to_f64(B.to_host_bits(got["vc_dev"]))
    assert_close(kc, ref["K"], "K cache after prefill + decode")
    assert_close(vc, ref["V"], "V cache after prefill + decode")


@pytest.mark.parametrize("separate", [False, True])
def test_prefill_layer_outputs_alone_with_a_tiny_residual(separate):
    """Residual stream scaled by 2^-10: R1 and R2 are then the reduced sub-layer outputs Z up to a negligible term, so
    the error bound is relative to Z (at full size with 0.02-std weights |Z| << |R| would hide an error in Z)."""
    cfg = _cfg(4, 2, 150, 8, 4 * 256, 0.5)
    d = make_inputs(cfg, seed=43, weight_std=0.05)
    d["R"] = I.f32_to_bf16_bits(I.bf16_bits_to_f32(d["R"]) * np.float32(2.0 ** -10))
    got = run_prefill(cfg, d, separate_reduce=separate)
    w, ref = oracle_prefill(cfg, d)
    assert np.abs(ref["R1"] - w["R"]).max() > 50 * np.abs(w["R"]).max()
    check_prefill(cfg, d, got, ref)
