"""Parity at the benchmark's full sizes (seed 0), in the launch configuration bench.py times: the whole oracle is run
on the host for each configuration (tens of seconds on the GPU machine) and every output tensor is compared."""
import numpy as np
import pytest

from paper_2506_19645_amd import inputs as I
from tests.test_gpu_attn import check_attn, check_attn_bwd, oracle_attn_block, oracle_attn_bwd, run_attn_block
from tests.test_gpu_block import check_mlp_block, oracle_mlp_block, run_mlp_block
from tests.test_gpu_decode import run_decode
from tests.test_gpu_prefill import check_prefill, oracle_prefill, run_prefill
from tests.util import assert_close, bits_to_f64, make_inputs, hs_of

pytestmark = pytest.mark.gpu


def test_config2_gpt_mlp_full_size():
    """h=2048 ffn=8192 GELU LayerNorm T=4 p=0.5, 8192 tokens, forward + backward."""
    cfg = I.C2
    d = make_inputs(cfg, seed=0)
    got = run_mlp_block(cfg, d)
    w, fwd, g = oracle_mlp_block(cfg, d)
    check_mlp_block(cfg, d, got, w, fwd, g)


@pytest.mark.parametrize("p", [1.0, 0.25, 0.0])
def test_config2_p_sweep_full_size_forward_backward(p):
    """The other points of the p sweep, forward + backward against the whole oracle (weight and norm-parameter
    gradients need every token), in the launch configuration the benchmark times."""
    cfg = I.C2.with_(p=p)
    d = make_inputs(cfg, seed=0)
    got = run_mlp_block(cfg, d)
    w, fwd, g = oracle_mlp_block(cfg, d)
    check_mlp_block(cfg, d, got, w, fwd, g)
    hs = hs_of(cfg)
    if hs > 0:
        for m in range(1, cfg.T):
            assert np.array_equal(got["Rp_bits"][m, :, :hs], got["Rp_bits"][0, :, :hs])


def test_config2_reduce_as_its_own_kernel_full_size_sampled_tokens():
    """The benchmark's sweep times the reduce as a kernel of its own (separate_reduce = 1): the same configuration,
    forward, against the oracle on a token sample (MLP rows are independent per token)."""
    cfg = I.C2
    d = make_inputs(cfg, seed=0, with_grads=False)
    got = run_mlp_block(cfg, d, backward=False, separate_reduce=True)
    rows = np.sort(np.random.default_rng(5).choice(cfg.tokens, size=96, replace=False))
    sub = {k: (v[:, rows] if k in ("X", "R") else v) for k, v in d.items()}
    small = cfg.with_(batch=1, seq=len(rows))
    w, fwd, _ = oracle_mlp_block(small, sub, backward=False)
    assert_close(got["Rp"][:, rows], fwd["Rp"], "Rp")
    assert_close(got["Xp"][:, rows], fwd["Xp"], "Xp")
    hs = hs_of(cfg)
    for m in range(1, cfg.T):
        assert np.array_equal(got["Rp_bits"][m, :, :hs], got["Rp_bits"][0, :, :hs])


def test_config3_llama_mlp_full_size():
    """h=4096 SwiGLU ffn=11008 RMSNorm T=8 (1376 columns per rank) p=0.5, 4096 tokens, forward + backward."""
    cfg = I.C3
    d = make_inputs(cfg, seed=0)
    got = run_mlp_block(cfg, d)
    w, fwd, g = oracle_mlp_block(cfg, d)
    check_mlp_block(cfg, d, got, w, fwd, g)


def test_config4_llama_attention_full_size():
    """h=4096, 32 heads of 128, RoPE, causal, seq 4096, T=8, p=0.5, forward + backward."""
    cfg = I.C4
    d = make_inputs(cfg, seed=0)
    got = run_attn_block(cfg, d, backward=True)
    w, fwd = oracle_attn_block(cfg, d)
    check_attn(cfg, d, got, fwd)
    check_attn_bwd(got, oracle_attn_bwd(cfg, w, fwd))


@pytest.mark.parametrize("p", [0.5, 1.0, 0.25, 0.0])
def test_config5_llama_decode_full_size(p):
    """batch 64, one new token, KV cache of 2048 positions per sequence, T=8, every p of the sweep."""
    from oracle import caat_oracle as O
    cfg = I.C5.with_(p=p)
    d = make_inputs(cfg, seed=0)
    got = run_decode(cfg, d)
    w = {k: O.widen_bf16(v, np.float32 if k in ("Kc", "Vc") else np.float64) for k, v in d.items()}   # caches: exact in fp32
    ref = O.decode_layer_fwd(w["R"], w, w["Kc"], w["Vc"], kv_len=cfg.kv_len, heads_per_rank=cfg.n_heads // cfg.T,
                             head_dim=cfg.head_dim, hs=hs_of(cfg))
    for name in ("X1", "H", "R1", "X2", "R2"):
        assert_close(got[name], ref[name], name)
    L = cfg.kv_len
    assert_close(bits_to_f64(got["Kc_bits"][:, :, :, L]), ref["k_new"], "k_new")
    assert_close(bits_to_f64(got["Vc_bits"][:, :, :, L]), ref["v_new"], "v_new")
    assert np.array_equal(got["Kc_bits"][:, :, :, :L], d["Kc"][:, :, :, :L])
    hs = hs_of(cfg)
    for m in range(1, cfg.T):
        assert np.array_equal(got["R2_bits"][m, :, :hs], got["R2_bits"][0, :, :hs])


def test_config5_sublayer_outputs_alone_with_a_tiny_residual():
    """At these weights |Z| << |R| (the attention output averages 2049 values, the weights have std 0.02), so R1 and R2
    say little about Z.  With the residual stream scaled by 2^-10 (exact in bf16; RMSNorm undoes it up to eps) R1 and R2
    ARE the reduced sub-layer outputs up to a negligible term, and the 2e-2 bound applies to Z itself, full size."""
    from oracle import caat_oracle as O
    cfg = I.C5
    d = make_inputs(cfg, seed=0)
    d["R"] = I.f32_to_bf16_bits(I.bf16_bits_to_f32(d["R"]) * np.float32(2.0 ** -10))
    got = run_decode(cfg, d)
    w = {k: O.widen_bf16(v, np.float32 if k in ("Kc", "Vc") else np.float64) for k, v in d.items()}
    ref = O.decode_layer_fwd(w["R"], w, w["Kc"], w["Vc"], kv_len=cfg.kv_len, heads_per_rank=cfg.n_heads // cfg.T,
                             head_dim=cfg.head_dim, hs=hs_of(cfg))
    assert np.sqrt(((ref["R1"] - w["R"]) ** 2).mean()) > 5 * np.sqrt((w["R"] ** 2).mean())
    for name in ("R1", "X2", "R2"):
        assert_close(got[name], ref[name], name)


def test_config6_prefill_layer_full_size_sampled_sequence():
    """Llama-7B decoder layer over 16 prompts of 2048 tokens (T=8, p=0.5): the GPU runs the whole batch; sequences are
    independent, so the oracle runs on one of them (all ranks) and is compared with that sequence's rows."""
    cfg = I.C6
    d = make_inputs(cfg, seed=0)
    got = run_prefill(cfg, d, keep=("H", "R1"))
    sq = 11
    rows = slice(sq * cfg.seq, (sq + 1) * cfg.seq)
    one = cfg.with_(batch=1)
    w, ref = oracle_prefill(one, dict(d, R=np.ascontiguousarray(d["R"][:, rows])))
    check_prefill(one, d, got, ref, rows=rows)
    assert_close(bits_to_f64(got["Kc_bits"][:, sq:sq + 1, :, :cfg.seq]), ref["K"], "K cache")
    assert_close(bits_to_f64(got["Vc_bits"][:, sq:sq + 1, :, :cfg.seq]), ref["V"], "V cache")
    hs = hs_of(cfg)
    for m in range(1, cfg.T):
        assert np.array_equal(got["R2_bits"][m, :, :hs], got["R2_bits"][0, :, :hs])


def test_config7_llama70b_gqa_prefill_layer_sampled_sequence():
    """Llama-2-70B dimensions (h=8192, 64 query heads, 8 key / value heads, ffn=28672), T=8, 8 prompts of 2048 tokens:
    the whole batch on the GPU, one sequence through the oracle."""
    cfg = I.C7
    d = make_inputs(cfg, seed=0)
    got = run_prefill(cfg, d, keep=("H",))
    sq = 5
    rows = slice(sq * cfg.seq, (sq + 1) * cfg.seq)
    one = cfg.with_(batch=1)
    w, ref = oracle_prefill(one, dict(d, R=np.ascontiguousarray(d["R"][:, rows])))
    check_prefill(one, d, got, ref, rows=rows)
    assert_close(bits_to_f64(got["Kc_bits"][:, sq:sq + 1, :, :cfg.seq]), ref["K"], "K cache")
    assert_close(bits_to_f64(got["Vc_bits"][:, sq:sq + 1, :, :cfg.seq]), ref["V"], "V cache")


@pytest.mark.parametrize("swi,p", [(False, 0.3), (True, 0.301)])
def test_ragged_shapes_on_the_big_persistent_tiles(swi, p):
    """Dimensions just past multiples of 256 (8264 tokens, h = 2056, 2056 columns per rank), large enough that the
    GEMMs take the 256 x 256 persistent tiles with several tiles per workgroup: every fused epilogue then meets edge
    tiles (rows and columns that do not exist) and, with hs = 616 (a multiple of 8) resp. 618 (not), both routes of
    the backward reduce.  Forward + backward against the whole oracle."""
    cfg = I.BlockConfig("ragged-big", I.KIND_MLP_SWIGLU if swi else I.KIND_MLP_GELU,
                        I.NORM_RMSNORM if swi else I.NORM_LAYERNORM, h=2056, T=4, p=p, batch=1, seq=8264, ffn=4 * 2056)
    assert hs_of(cfg) == (618 if swi else 616)
    d = make_inputs(cfg, seed=3)
    got = run_mlp_block(cfg, d)
    w, fwd, g = oracle_mlp_block(cfg, d)
    check_mlp_block(cfg, d, got, w, fwd, g)
