"""GPU parity of the single-device serving mode (Sec. 3.2, logical ranks: the partial channel-reduce becomes a local
summation): with reduce_in_gemm the shared channels come from one GEMM whose contraction runs over all ranks.  The
oracle is the same as for the default path: the result is the same sum, only accumulated without intermediate rounding."""
import numpy as np
import pytest

from oracle import caat_oracle as O
from paper_2506_19645_amd import inputs as I
from tests.test_gpu_attn import _cfg as attn_cfg, check_attn, oracle_attn_block, run_attn_block
from tests.test_gpu_block import _cfg as mlp_cfg, check_mlp_block, oracle_mlp_block, run_mlp_block
from tests.test_gpu_decode import _cfg as dec_cfg, run_decode
from tests.test_gpu_prefill import _cfg as pre_cfg, check_prefill, oracle_prefill, run_prefill
from tests.util import assert_close, make_inputs, hs_of

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("swi", [False, True])
@pytest.mark.parametrize("T,n,h,ffn,p,scale", [
    (2, 40, 64, 256, 0.5, 1.0),                 # hs = 32
    (3, 300, 264, 3 * 344, 0.5, 1.0),           # hs = 132: not a multiple of 8 -> the default path is taken
    (3, 300, 256, 3 * 344, 0.25, 1.0),          # T = 3, contraction of 3 x 344 with a ragged last stage per rank
    (4, 515, 512, 4 * 520, 0.25, 2.0),          # private channel scaling
    (2, 129, 256, 1024, 1.0, 1.0),              # p = 1: only the shared GEMM runs
    (2, 129, 256, 1024, 0.0, 1.0),              # p = 0: only the private GEMM runs
    (8, 300, 1024, 8 * 136, 0.5, 1.0),          # T = 8, 136 columns per rank (4 stages + tail of 8)
])
def test_mlp_block_reduce_in_gemm(swi, T, n, h, ffn, p, scale):
    cfg = mlp_cfg(swi, T, n, h, ffn, p, scale)
    d = make_inputs(cfg, seed=51, weight_std=0.05)
    got = run_mlp_block(cfg, d, reduce_in_gemm=True)      # backward runs on the forward's saved tensors as usual
    w, fwd, g = oracle_mlp_block(cfg, d)
    check_mlp_block(cfg, d, got, w, fwd, g)
    # against the default path: private channels are computed by the same arithmetic -> same bits
    ref = run_mlp_block(cfg, d, backward=False)
    assert np.array_equal(got["Rp_bits"][:, :, hs_of(cfg):], ref["Rp_bits"][:, :, hs_of(cfg):])


def test_attention_block_reduce_in_gemm():
    cfg = attn_cfg(2, 2, 200, 4, 0.5)
    d = make_inputs(cfg, seed=52, with_grads=False, weight_std=0.05)
    got = run_attn_block(cfg, d, reduce_in_gemm=True)
    w, fwd = oracle_attn_block(cfg, d)
    check_attn(cfg, d, got, fwd)


@pytest.mark.parametrize("kv_heads", [0, 2])
def test_decode_layer_reduce_in_gemm(kv_heads):
    cfg = dec_cfg(2, 37, 8, 2 * 344, 150, 0.5, kv_heads)
    d = make_inputs(cfg, seed=53, weight_std=0.05)
    got = run_decode(cfg, d, reduce_in_gemm=True)
    w = {k: O.widen_bf16(v) for k, v in d.items()}
    ref = O.decode_layer_fwd(w["R"], w, w["Kc"], w["Vc"], kv_len=cfg.kv_len, heads_per_rank=cfg.n_heads // cfg.T,
                             head_dim=128, hs=hs_of(cfg), kv_heads_per_rank=cfg.kv_heads // cfg.T)
    for name in ("R1", "X2", "R2"):
        assert_close(got[name], ref[name], name)
    for m in range(1, cfg.T):
        assert np.array_equal(got["R2_bits"][m, :, :hs_of(cfg)], got["R2_bits"][0, :, :hs_of(cfg)])


def test_prefill_layer_reduce_in_gemm():
    cfg = pre_cfg(4, 2, 200, 4, 4 * 344, 0.25)
    d = make_inputs(cfg, seed=54, weight_std=0.05)
    got = run_prefill(cfg, d, reduce_in_gemm=True)
    w, ref = oracle_prefill(cfg, d)
    check_prefill(cfg, d, got, ref)
    for m in range(1, cfg.T):
        assert np.array_equal(got["R2_bits"][m, :, :hs_of(cfg)], got["R2_bits"][0, :, :hs_of(cfg)])


# ---------------------------------------------------------------------------------------------------------
# De-duplicated residual stream: the shared channels are stored once ([n, hs]) instead of T identical copies.
def _run_mlp_dedup(cfg, d):
    import torch
    from paper_2506_19645_amd import binding as B
    from tests.util import pack_dedup, unpack_dedup
    swi = cfg.kind == I.KIND_MLP_SWIGLU
    desc = B.make_desc(cfg, reduce_in_gemm=True, dedup_shared=True)
    T, n, h, hs = cfg.T, cfg.tokens, cfg.h, hs_of(cfg)
    w0 = B.to_device(np.concatenate([d["Wg"], d["Wu"]], axis=1) if swi else d["A"])
    weights = [w0, B.to_device(d["B"]), B.to_device(d["gamma"]), B.to_device(d["beta"]) if "beta" in d else None]
    x = B.to_device(d["X"])
    r = B.to_device(pack_dedup(d["R"], hs))
    r_out, x_out = torch.zeros_like(r), torch.empty_like(x)
    ws = torch.zeros(B.workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    B.block_fwd(desc, weights, x, r, r_out, x_out, ws)
    torch.cuda.synchronize()
    return unpack_dedup(B.to_host_bits(r_out), T, n, h, hs), B.to_host_bits(x_out)


@pytest.mark.parametrize("swi,T,n,h,ffn,p", [
    (False, 2, 129, 256, 1024, 0.5),
    (True, 4, 515, 512, 4 * 520, 0.25),
    (True, 3, 300, 256, 3 * 344, 1.0),      # everything shared: the private block is empty
    (False, 2, 200, 256, 1024, 0.0),        # nothing shared: the layout is the ordinary one
])
def test_mlp_block_dedup_shared_layout(swi, T, n, h, ffn, p):
    cfg = mlp_cfg(swi, T, n, h, ffn, p, 1.0)
    d = make_inputs(cfg, seed=55, weight_std=0.05)
    rp_bits, xp_bits = _run_mlp_dedup(cfg, d)
    ref = run_mlp_block(cfg, d, backward=False, reduce_in_gemm=True)   # same arithmetic, T copies of the shared columns
    assert np.array_equal(rp_bits, ref["Rp_bits"])
    assert np.array_equal(xp_bits, ref["Xp_bits"])
    w, fwd, _ = oracle_mlp_block(cfg, d, backward=False)
    from tests.util import bits_to_f64
    assert_close(bits_to_f64(rp_bits), fwd["Rp"], "Rp")
    assert_close(bits_to_f64(xp_bits), fwd["Xp"], "Xp")


def test_prefill_layer_dedup_shared_layout():
    import torch
    from paper_2506_19645_amd import binding as B
    from tests.test_gpu_prefill import layer_weights
    from tests.util import bits_to_f64, pack_dedup, unpack_dedup
    cfg = pre_cfg(4, 2, 200, 8, 4 * 344, 0.25, kv_heads=4)
    d = make_inputs(cfg, seed=56, weight_std=0.05)
    T, n, h, hs = cfg.T, cfg.tokens, cfg.h, hs_of(cfg)
    desc = B.make_desc(cfg, reduce_in_gemm=True, dedup_shared=True)
    r = B.to_device(pack_dedup(d["R"], hs))
    r_out = torch.zeros_like(r)
    kc = torch.zeros((T, cfg.batch, cfg.kv_heads // T, desc.kv_cap, 128), dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    ws = torch.zeros(B.workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    B.block_fwd(desc, layer_weights(d), None, r, r_out, None, ws, kv_k=kc, kv_v=vc)
    torch.cuda.synchronize()
    r2_bits = unpack_dedup(B.to_host_bits(r_out), T, n, h, hs)
    ref_gpu = run_prefill(cfg, d, reduce_in_gemm=True)
    assert np.array_equal(r2_bits, ref_gpu["R2_bits"])
    assert np.array_equal(B.to_host_bits(kc), ref_gpu["Kc_bits"])
    w, ref = oracle_prefill(cfg, d)
    assert_close(bits_to_f64(r2_bits), ref["R2"], "R2")


def test_dedup_layout_is_refused_where_it_cannot_exist():
    from paper_2506_19645_amd import binding as B
    cfg = mlp_cfg(False, 2, 129, 256, 1024, 0.5, 1.0)
    assert B.workspace_bytes(B.make_desc(cfg, reduce_in_gemm=False, dedup_shared=True)) == 0     # needs the reduce in the GEMM
    assert B.workspace_bytes(B.make_desc(cfg.with_(p=0.3), reduce_in_gemm=True, dedup_shared=True)) == 0   # hs = 76
    assert B.workspace_bytes(B.make_desc(cfg.with_(seq=64), reduce_in_gemm=True, dedup_shared=True)) == 0  # 64 tokens
    assert B.workspace_bytes(B.make_desc(cfg, reduce_in_gemm=True, dedup_shared=True)) > 0
