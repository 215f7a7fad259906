"""GPU parity of the decode layer (one new token per sequence over a KV cache) against the CPU oracle."""
import numpy as np
import pytest

from oracle import caat_oracle as O
from paper_2506_19645_amd import binding as B
from paper_2506_19645_amd import inputs as I
from tests.util import assert_close, bits_to_f64, make_inputs, hs_of

pytestmark = pytest.mark.gpu


def run_decode(cfg, d, reduce_in_gemm=False, separate_reduce=False):
    import torch
    desc = B.make_desc(cfg, reduce_in_gemm=reduce_in_gemm, separate_reduce=separate_reduce)
    T, b, h, hd = cfg.T, cfg.batch, cfg.h, cfg.hd_r
    weights = [B.to_device(d["gamma_attn"]), B.to_device(d["Wqkv"]), B.to_device(d["Wo"]), B.to_device(d["gamma"]),
               B.to_device(np.concatenate([d["Wg"], d["Wu"]], axis=1)), B.to_device(d["B"])]
    r = B.to_device(d["R"])
    kc, vc = B.to_device(d["Kc"]), B.to_device(d["Vc"])
    r_out = torch.empty_like(r)
    ws = torch.zeros(B.workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    B.block_fwd(desc, weights, None, r, r_out, None, ws, kv_k=kc, kv_v=vc)
    torch.cuda.synchronize()
    L = B.workspace_layout(desc)

    def ws_bf16(off, nbytes, shape):
        return bits_to_f64(ws[off:off + nbytes].view(torch.int16).cpu().numpy().view(np.uint16).reshape(shape))

    return {"R2": bits_to_f64(B.to_host_bits(r_out)), "R2_bits": B.to_host_bits(r_out),
            "X1": ws_bf16(L.off_X1, L.bytes_X1, (T, b, h)), "H": ws_bf16(L.off_H, L.bytes_H, (T, b, hd)),
            "R1": ws_bf16(L.off_R1, L.bytes_R1, (T, b, h)), "X2": ws_bf16(L.off_X2, L.bytes_X2, (T, b, h)),
            "R1_bits": ws[L.off_R1:L.off_R1 + L.bytes_R1].view(torch.int16).cpu().numpy().view(np.uint16).reshape(T, b, h),
            "Kc_bits": B.to_host_bits(kc), "Vc_bits": B.to_host_bits(vc)}


def _cfg(T, b, heads, ffn, L, p, kv_heads=0, scale=1.0):
    return I.BlockConfig("dec", I.KIND_DECODE, I.NORM_RMSNORM, h=heads * 128, T=T, p=p, batch=b, seq=1, ffn=ffn,
                         n_heads=heads, head_dim=128, kv_len=L, n_kv_heads=kv_heads, private_scale=scale)


def oracle_decode(cfg, d):
    w = {k: O.widen_bf16(v) for k, v in d.items()}
    return O.decode_layer_fwd(w["R"], w, w["Kc"], w["Vc"], kv_len=cfg.kv_len, heads_per_rank=cfg.n_heads // cfg.T,
                              head_dim=cfg.head_dim, hs=hs_of(cfg), eps=cfg.eps, private_scale=cfg.private_scale,
                              rope_base=cfg.rope_base, kv_heads_per_rank=cfg.kv_heads // cfg.T)


@pytest.mark.parametrize("T,b,heads,ffn,L,p,kv_heads,scale", [
    (2, 3, 4, 2 * 344, 37, 0.5, 0, 1.0),      # fewer keys than one 64-key sweep, ragged ffn shard
    (2, 64, 4, 2 * 256, 300, 0.25, 0, 1.0),   # the benchmark's batch, several sweeps + tail
    (4, 5, 4, 4 * 128, 0, 1.0, 0, 1.0),       # empty cache: the token attends to itself only
    (1, 2, 2, 256, 129, 0.0, 0, 1.0),
    (2, 5, 8, 2 * 256, 200, 0.5, 2, 1.0),     # grouped-query attention: 4 query heads per key / value head
    (2, 3, 8, 2 * 256, 70, 0.5, 4, 1.0),      # two groups per rank
    (2, 4, 4, 2 * 256, 50, 0.3, 0, 1.0),      # hs = 153: not a multiple of 8, so the reduce and the norm stay two kernels
    (8, 6, 8, 8 * 128, 90, 0.5, 0, 1.0),      # tensor-parallel degree 8 through the one-launch reduce + norm
    (4, 7, 4, 4 * 128, 61, 0.5, 0, 2.0),      # private channel scaling sqrt(T) (Sec. 4) in both halves of the layer
    (2, 5, 4, 2 * 256, 40, 0.0, 0, 2.0 ** 0.5),   # the same at p = 0: every channel private and scaled
    (16, 3, 32, 16 * 128, 70, 0.5, 0, 1.0),   # tensor-parallel degree 16 (Sec. 5's largest): 32 heads, 2 per rank
    (16, 2, 32, 16 * 136, 20, 0.3, 0, 4.0),   # T = 16, hs not a multiple of 8 (two-kernel route), scaling sqrt(T)
])
def test_decode_layer(T, b, heads, ffn, L, p, kv_heads, scale):
    cfg = _cfg(T, b, heads, ffn, L, p, kv_heads, scale)
    d = make_inputs(cfg, seed=31, weight_std=0.05 if cfg.h < 4096 else 0.02)   # h = 4096: scores stay O(1), as in the benchmark
    got = run_decode(cfg, d)
    ref = oracle_decode(cfg, d)
    assert_close(got["X1"], ref["X1"], "X1")
    assert_close(got["H"], ref["H"], "H")
    assert_close(got["R1"], ref["R1"], "R1")
    assert_close(got["X2"], ref["X2"], "X2")
    assert_close(got["R2"], ref["R2"], "R2")
    # the new token's rotated k and its v were appended at position L; every older cache row keeps its bits
    assert_close(bits_to_f64(got["Kc_bits"][:, :, :, L]), ref["k_new"], "k_new")
    assert_close(bits_to_f64(got["Vc_bits"][:, :, :, L]), ref["v_new"], "v_new")
    assert np.array_equal(got["Kc_bits"][:, :, :, :L], d["Kc"][:, :, :, :L])
    assert np.array_equal(got["Vc_bits"][:, :, :, :L], d["Vc"][:, :, :, :L])
    hs = hs_of(cfg)
    if hs > 0 and T > 1 and np.array_equal(d["R"][0, :, :hs], d["R"][-1, :, :hs]):
        for m in range(1, T):
            assert np.array_equal(got["R2_bits"][m, :, :hs], got["R2_bits"][0, :, :hs])
            assert np.array_equal(got["R1_bits"][m, :, :hs], got["R1_bits"][0, :, :hs])


@pytest.mark.parametrize("separate", [False, True])
def test_decode_layer_outputs_alone_with_a_tiny_residual(separate):
    """With the residual stream scaled down by 2^-10 (RMSNorm does not care, up to eps) both R1 and R2 are dominated by
    the reduced sub-layer outputs Z, so the relative error is measured against Z itself and not hidden behind
    R ~ N(0,1); run through both routes (one-launch reduce + norm, and the reduce as a kernel of its own)."""
    cfg = _cfg(4, 9, 8, 4 * 256, 150, 0.5)
    d = make_inputs(cfg, seed=33, weight_std=0.05)
    d["R"] = I.f32_to_bf16_bits(I.bf16_bits_to_f32(d["R"]) * np.float32(2.0 ** -10))     # exact: a power of two
    got = run_decode(cfg, d, separate_reduce=separate)
    ref = oracle_decode(cfg, d)
    assert np.abs(ref["R1"] - O.widen_bf16(d["R"])).max() > 50 * np.abs(O.widen_bf16(d["R"])).max()
    for name in ("R1", "X2", "R2"):
        assert_close(got[name], ref[name], name)
    hs = hs_of(cfg)
    for m in range(1, cfg.T):
        assert np.array_equal(got["R2_bits"][m, :, :hs], got["R2_bits"][0, :, :hs])
