"""CPU-side checks of the C ABI: the library loads, exports every symbol include/caat.h declares, and the
host-side validation returns error codes before anything is launched (no compute here)."""
import ctypes as C
import os
import re

import pytest

from paper_2506_19645_amd import binding as B
from paper_2506_19645_amd import inputs as I

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared(path):
    txt = open(os.path.join(ROOT, *path)).read()
    txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
    return sorted(set(re.findall(r"\b(caat_[a-z0-9_]+)\s*\(", txt)))


def test_library_exports_every_declared_symbol():
    names = _declared(("include", "caat.h"))
    assert set(names) == set(B.EXPORTS)
    tools = _declared(("paper_2506_19645_amd", "csrc", "caat_tools.h"))     # measuring tools, outside the method's ABI
    assert set(tools) == set(B.TOOL_EXPORTS) and not set(tools) & set(names)
    L = B.lib()
    for n in names + tools:
        assert getattr(L, n) is not None


def test_shared_channels_matches_floor():
    assert B.shared_channels(768, 0.5) == 384
    assert B.shared_channels(768, 0.3) == 230
    assert B.shared_channels(4096, 0.703125) == 2880
    assert B.shared_channels(4096, 0.7) == 2867
    assert B.shared_channels(4096, 1.0) == 4096 and B.shared_channels(4096, 0.0) == 0
    for bad in (-0.01, 1.01, float("nan")):
        assert B.shared_channels(16, bad) == -1
    # the library's count (what the GPU descriptor gets) against the oracle's (what the oracle calls get): two
    # independent implementations of Eq. A3's floor(h*p), over the benchmark shapes and a sweep of awkward p
    from oracle import caat_oracle as O
    for cfg in I.CONFIGS.values():
        for p in (1.0, 0.5, 0.25, 0.0, 0.3, 0.301, 0.7, 1.0 / 3.0, 90.0 / 128.0, 1e-9, 1.0 - 1e-12):
            assert B.shared_channels(cfg.h, p) == O.shared_channels(cfg.h, p)


def test_status_strings():
    seen = {B.status_string(s) for s in range(8)}
    assert len(seen) == 8 and B.status_string(0) == "ok"


def test_validation_errors_before_launch():
    # host-side checks only: all pointers are fake but validation fails before they are used
    fake = 0x1000
    assert B.partial_sync(None, None, fake, 2, 4, 16, 8, stream=0, check=False) == B.EINVAL
    assert B.partial_sync(fake, None, fake, 0, 4, 16, 8, stream=0, check=False) == B.EINVAL
    assert B.partial_sync(fake, None, fake, 2, 4, 16, 17, stream=0, check=False) == B.ESHAPE
    assert B.partial_sync(fake, None, fake, 2, 4, 12, 4, stream=0, check=False) == B.ESHAPE      # h % 8
    assert B.partial_sync(fake + 2, None, fake, 2, 4, 16, 8, stream=0, check=False) == B.EALIGN
    assert B.partial_sync(fake, None, fake, 2, 4, 16, 8, private_scale=float("nan"), stream=0, check=False) == B.EINVAL
    assert B.norm_fwd(fake, fake, None, fake, fake, fake, B.LAYERNORM, 2, 4, 16, 1e-5, stream=0, check=False) == B.EINVAL
    assert B.norm_fwd(fake, fake, None, fake, None, fake, 7, 2, 4, 16, 1e-5, stream=0, check=False) == B.EINVAL
    # the entry point that allocates nothing refuses what its fixed 16 MiB scratch cannot hold, before any launch:
    # h = 8192 needs 8 h bytes per partial row of 8 token rows, so more than 2048 rows do not fit
    st = lambda T, n, h: B.norm_bwd_static(fake, None, fake, fake, None, fake, fake, None, fake, None, B.RMSNORM, T, n, h, 0,
                                           1.0, stream=0, check=False)
    assert st(1, 2056, 8192) == B.ESCRATCH and st(8, 4096, 8192) == B.ESCRATCH
    assert B.norm_bwd_workspace_bytes(1, 2048, 8192) == 16 << 20 and B.norm_bwd_workspace_bytes(16, 1 << 20, 4096) == 16 << 20
    assert st(1, 8, 8200) == B.ESHAPE and st(0, 8, 64) == B.EINVAL
    assert B.gemm_bf16(fake, fake, fake, B.GEMM_NT, 1, 8, 12, 8, 8, 8, 16, 0, 0, 0, stream=0, check=False) == B.ESHAPE
    assert B.gemm_bf16(fake, fake, fake, 5, 1, 8, 8, 8, 8, 8, 8, 0, 0, 0, stream=0, check=False) == B.EINVAL
    assert B.gemm_bf16(fake, fake, fake + 4, B.GEMM_NT, 1, 8, 8, 8, 8, 8, 8, 0, 0, 0, stream=0, check=False) == B.EALIGN


def test_descriptor_validation_and_workspace():
    d = B.make_desc(I.C1)
    assert B.workspace_bytes(d) > 0
    L = B.workspace_layout(d)
    assert L.total_bytes == B.workspace_bytes(d)
    assert L.bytes_P == 2 * 256 * 1536 * 2 and L.bytes_Y == L.bytes_P and L.bytes_dZt == 2 * 256 * 768 * 2
    d3 = B.make_desc(I.C3)
    L3 = B.workspace_layout(d3)
    assert L3.bytes_P == 2 * L3.bytes_Y                      # gate|up pre-activations
    bad = B.make_desc(I.C1)
    bad.ffn = 3073
    assert B.workspace_bytes(bad) == 0
    bad = B.make_desc(I.C1)
    bad.hs = 769
    assert B.workspace_bytes(bad) == 0
    bad = B.make_desc(I.C1)
    bad.T = 0
    assert B.workspace_bytes(bad) == 0
    fake = 0x1000
    w = [fake, fake, fake, fake]
    assert B.block_fwd(d, w, fake, fake, fake, fake, None, stream=0, check=False) == B.EINVAL       # no workspace
    bad = B.make_desc(I.C1)
    bad.hs = -1
    assert B.block_fwd(bad, w, fake, fake, fake, fake, None, stream=0, check=False) == B.ESHAPE


def test_no_fallback_when_library_missing(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError):
        B.lib()


def test_descriptor_validation_of_the_attention_and_serving_fields():
    ok = I.BlockConfig("a", I.KIND_ATTN, I.NORM_RMSNORM, h=1024, T=2, p=0.5, batch=1, seq=256, n_heads=8, head_dim=128,
                       n_kv_heads=4)
    assert B.workspace_bytes(B.make_desc(ok)) > 0
    assert B.workspace_bytes(B.make_desc(ok.with_(n_kv_heads=3))) == 0       # 8 % 3
    assert B.workspace_bytes(B.make_desc(ok.with_(n_kv_heads=1))) == 0       # fewer key / value heads than ranks
    assert B.workspace_bytes(B.make_desc(ok.with_(T=3))) == 0                # heads do not divide over the ranks
    d = B.make_desc(ok)
    d.reduce_in_gemm = 2
    assert B.workspace_bytes(d) == 0
    d = B.make_desc(ok, reduce_in_gemm=True, dedup_shared=True)
    assert B.workspace_bytes(d) > 0
    d.reduce_in_gemm = 0
    assert B.workspace_bytes(d) == 0                                         # stored-once layout needs the reduce in the GEMM
    L = B.workspace_layout(B.make_desc(ok))
    qw = (4 + 2 * 2) * 128
    assert L.bytes_Q == 2 * 256 * qw * 2 and L.bytes_dP == L.bytes_Q and L.bytes_dH == 2 * 256 * 512 * 2
    assert L.bytes_stats == 2 * 4 * 2 * 256 * 4
    pre = I.C6
    assert B.workspace_bytes(B.make_desc(pre)) > 0
    assert B.workspace_bytes(B.make_desc(pre, kv_cap=pre.seq - 1)) > 0       # capacity is checked at the call, not here
