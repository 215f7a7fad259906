"""Edge cases of the C ABI on the GPU: empty inputs, error paths that must leave outputs untouched, extreme shared
channel counts, the widest supported hidden size, and the per-launch timing tool."""
import numpy as np
import pytest

from paper_2506_19645_amd import binding as B
from paper_2506_19645_amd import inputs as I
from tests.test_gpu_attn import _cfg as attn_cfg, check_attn, check_attn_bwd, oracle_attn_block, oracle_attn_bwd, run_attn_block
from tests.test_gpu_block import _cfg as mlp_cfg, check_mlp_block, oracle_mlp_block, run_mlp_block
from tests.util import make_inputs, hs_of

pytestmark = pytest.mark.gpu


def _mlp_buffers(cfg, d, sentinel=0x7FC0):
    import torch
    w = [B.to_device(d["A"]), B.to_device(d["B"]), B.to_device(d["gamma"]), B.to_device(d["beta"])]
    x, r = B.to_device(d["X"]), B.to_device(d["R"])
    fill = lambda t: torch.full_like(t.view(torch.int16), sentinel).view(torch.bfloat16)
    return w, x, r, fill(x), fill(x)


def test_zero_tokens_is_a_no_op():
    import torch
    cfg = mlp_cfg(False, 2, 8, 64, 256, 0.5)
    d = make_inputs(cfg, seed=61)
    w, x, r, r_out, x_out = _mlp_buffers(cfg, d)
    desc = B.make_desc(cfg)
    desc.tokens, desc.seq = 0, 0
    ws = torch.zeros(max(B.workspace_bytes(desc), 256), dtype=torch.uint8, device="cuda")
    assert B.block_fwd(desc, w, x, r, r_out, x_out, ws, check=False) == B.OK
    dw = [torch.zeros_like(w[0]), torch.zeros_like(w[1])]
    dg, db = torch.zeros(cfg.h, device="cuda"), torch.zeros(cfg.h, device="cuda")
    assert B.block_bwd(desc, w, x, r_out, ws, x, x, x_out, r_out, dw, dg, db, check=False) == B.OK
    torch.cuda.synchronize()
    assert (B.to_host_bits(r_out) == 0x7FC0).all() and (B.to_host_bits(x_out) == 0x7FC0).all()
    assert B.partial_sync(x, None, x, 2, 0, 64, 32, check=False) == B.OK


def test_errors_leave_outputs_untouched():
    import torch
    cfg = mlp_cfg(False, 2, 40, 64, 256, 0.5)
    d = make_inputs(cfg, seed=62)
    w, x, r, r_out, x_out = _mlp_buffers(cfg, d)
    desc = B.make_desc(cfg)
    need = B.workspace_bytes(desc)
    small = torch.zeros(need - 256, dtype=torch.uint8, device="cuda")
    assert B.block_fwd(desc, w, x, r, r_out, x_out, small, check=False) == B.EWORKSPACE
    ws = torch.zeros(need, dtype=torch.uint8, device="cuda")
    bad = B.make_desc(cfg)
    bad.hs = cfg.h + 1
    assert B.block_fwd(bad, w, x, r, r_out, x_out, ws, check=False) == B.ESHAPE
    assert B.block_fwd(desc, w, x, r.data_ptr() + 2, r_out, x_out, ws, check=False) == B.EALIGN
    assert B.block_fwd(desc, [w[0], None, w[2], w[3]], x, r, r_out, x_out, ws, check=False) == B.EINVAL
    torch.cuda.synchronize()
    assert (B.to_host_bits(r_out) == 0x7FC0).all() and (B.to_host_bits(x_out) == 0x7FC0).all()
    with pytest.raises(B.CaatError) as ei:
        B.block_fwd(desc, w, x, r, r_out, x_out, small)
    assert ei.value.status == B.EWORKSPACE and "workspace" in str(ei.value)


def test_unsupported_requests_are_refused():
    import torch
    dec = I.BlockConfig("d", I.KIND_DECODE, I.NORM_RMSNORM, h=256, T=2, p=0.5, batch=2, seq=1, ffn=512, n_heads=2,
                        head_dim=128, kv_len=3)
    desc = B.make_desc(dec)
    fake = torch.zeros(1 << 16, dtype=torch.bfloat16, device="cuda")
    ws = torch.zeros(B.workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    w6 = [fake] * 6
    g = torch.zeros(256, device="cuda")
    assert B.block_bwd(desc, w6, fake, fake, ws, fake, fake, fake, fake, [fake, fake], g, None, check=False) == B.EUNSUPPORTED
    d64 = I.BlockConfig("a", I.KIND_ATTN, I.NORM_RMSNORM, h=128, T=2, p=0.5, batch=1, seq=8, n_heads=2, head_dim=64)
    desc64 = B.make_desc(d64)
    ws64 = torch.zeros(max(B.workspace_bytes(desc64), 256), dtype=torch.uint8, device="cuda")
    assert B.block_fwd(desc64, [fake] * 4, fake, fake, fake, fake, ws64, check=False) == B.EUNSUPPORTED   # head_dim != 128
    ln = B.make_desc(dec)
    ln.norm = B.LAYERNORM
    assert B.block_fwd(ln, w6, None, fake, fake, None, ws, kv_k=fake, kv_v=fake, check=False) == B.EUNSUPPORTED


@pytest.mark.parametrize("hs", [1, 7, 8, 2047, 2048 - 8])
def test_extreme_shared_channel_counts(hs):
    """One shared channel, a partial first group, all but one channel shared: the case split of Eq. A3 at its edges."""
    cfg = mlp_cfg(False, 2, 70, 2048, 512, hs / 2048.0)
    assert hs_of(cfg) == hs
    d = make_inputs(cfg, seed=63, weight_std=0.05)
    got = run_mlp_block(cfg, d)
    w, fwd, g = oracle_mlp_block(cfg, d)
    check_mlp_block(cfg, d, got, w, fwd, g)


@pytest.mark.parametrize("swi", [False, True])
def test_widest_hidden_size(swi):
    """h = 8192 is the widest row the norm kernels take; T = 2, ragged token count."""
    cfg = mlp_cfg(swi, 2, 77, 8192, 2 * 264, 0.5)
    d = make_inputs(cfg, seed=64, weight_std=0.02)
    got = run_mlp_block(cfg, d)
    w, fwd, g = oracle_mlp_block(cfg, d)
    check_mlp_block(cfg, d, got, w, fwd, g)


def test_single_rank_partial_sync_is_identity_plus_residual():
    cfg = mlp_cfg(True, 1, 129, 256, 512, 0.5)
    d = make_inputs(cfg, seed=65, weight_std=0.05)
    got = run_mlp_block(cfg, d)
    w, fwd, g = oracle_mlp_block(cfg, d)
    check_mlp_block(cfg, d, got, w, fwd, g)
    other = run_mlp_block(cfg.with_(p=0.0), d, backward=False)
    assert np.array_equal(got["Rp_bits"], other["Rp_bits"])       # with one rank, p does not matter


def test_attention_one_past_a_block_boundary():
    cfg = attn_cfg(2, 2, 129, 2, 0.5)
    d = make_inputs(cfg, seed=66, with_grads=True, weight_std=0.05)
    got = run_attn_block(cfg, d, backward=True)
    w, fwd = oracle_attn_block(cfg, d)
    check_attn(cfg, d, got, fwd)
    check_attn_bwd(got, oracle_attn_bwd(cfg, w, fwd))


@pytest.mark.parametrize("separate", [False, True])
def test_profile_records_every_launch(separate):
    cfg = mlp_cfg(False, 2, 40, 64, 256, 0.5)
    d = make_inputs(cfg, seed=67)
    B.profile_reset()
    B.profile_enable(True)
    try:
        run_mlp_block(cfg, d, separate_reduce=separate)
    finally:
        B.profile_enable(False)
    rec = B.profile_records()
    names = [n for n, _ in rec]
    # forward: reduce + residual + norm in one launch, backward: norm backward + reduce in one launch, unless the
    # caller asks for the reduce as a kernel of its own
    mid = ["partial_sync_fwd", "norm_fwd", "norm_bwd", "partial_sync_bwd"] if separate else ["partial_sync_norm_fwd", "norm_bwd_sync"]
    assert names == ["gemm_nt_gelu_fwd", "gemm_nt_rowpar"] + mid + ["gemm_nn_gelu_bwd", "gemm_tn_wgrad", "gemm_nn_dgrad",
                                                                   "gemm_tn_wgrad"]
    assert all(ms > 0.0 for _, ms in rec)
    B.profile_reset()
    assert B.profile_records() == []


def test_hbm_probe_modes():
    """The measuring tool: every mode runs, the copy modes copy, bad arguments are refused before any launch."""
    import torch
    n = (1 << 20) + 4096                      # not a multiple of the per-workgroup piece
    src = torch.arange(n, dtype=torch.int64, device="cuda").to(torch.uint8)
    for mode in (0, 1, 2):
        B.hbm_probe(src, torch.zeros(16, dtype=torch.uint8, device="cuda"), n, mode)
    for mode in (3, 4):
        dst = torch.zeros(n, dtype=torch.uint8, device="cuda")
        B.hbm_probe(src, dst, n, mode)
        torch.cuda.synchronize()
        assert torch.equal(dst, src), mode
    L = B.lib()
    assert L.caat_hbm_probe(B._ptr(src), None, n, 3, None) == 1        # copy without a destination
    assert L.caat_hbm_probe(B._ptr(src), None, n, 7, None) == 1        # unknown mode
    assert L.caat_hbm_probe(B._ptr(src), None, n - 8, 0, None) == 2    # size not a multiple of 16
