"""Helpers shared by the tests: error metrics and host<->device marshalling (no method arithmetic)."""
import numpy as np

from oracle import caat_oracle as O
from paper_2506_19645_amd import inputs as I

TOL = 2e-2   # relative error bound of the benchmark definition (bf16 storage, fp32 accumulation)


def hs_of(cfg) -> int:
    """Number of shared channels the ORACLE derives from (h, p) (Sec. 3, Eq. A3).  The GPU descriptor gets its own
    count from the library's caat_shared_channels (binding.make_desc); the two are cross-checked in test_abi."""
    return O.shared_channels(cfg.h, float(cfg.p))


def make_inputs(cfg, **kw):
    """inputs.make_inputs with the residual stream's rank-equal leading columns set to the oracle's shared-channel
    count unless the test says otherwise (the generator itself knows nothing about the method)."""
    kw.setdefault("hs_struct", hs_of(cfg))
    return I.make_inputs(cfg, **kw)


def rel_errs(got: np.ndarray, want: np.ndarray):
    """(max-norm relative error, L2 relative error) of got against want."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    den_max = max(float(np.abs(want).max()), 1e-30)
    den_l2 = max(float(np.sqrt((want * want).sum())), 1e-30)
    d = got - want
    return float(np.abs(d).max()) / den_max, float(np.sqrt((d * d).sum())) / den_l2


def assert_close(got, want, name, tol=TOL):
    assert np.all(np.isfinite(np.asarray(got, dtype=np.float64))), name + ": non-finite output"
    emax, el2 = rel_errs(got, want)
    assert emax <= tol and el2 <= tol, "%s: max-rel %.3e l2-rel %.3e > %.1e" % (name, emax, el2, tol)
    return emax, el2


def bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return I.bf16_bits_to_f32(bits).astype(np.float64)


def f64_to_bits(a: np.ndarray) -> np.ndarray:
    return I.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def ulp_distance_bf16(a_bits: np.ndarray, b_bits: np.ndarray) -> np.ndarray:
    """Distance in bf16 units-in-the-last-place between two bit-pattern arrays (sign-magnitude aware)."""
    def key(u):
        u = u.astype(np.int32)
        return np.where(u & 0x8000, -(u & 0x7FFF), u & 0x7FFF)
    return np.abs(key(a_bits) - key(b_bits))


def pack_dedup(bits, hs):
    """[T, n, h] residual-stream bit patterns whose first hs columns are equal on all ranks -> the de-duplicated
    layout: [n, hs] once, then the private columns [T, n, h - hs], flattened into one buffer."""
    assert all(np.array_equal(bits[m, :, :hs], bits[0, :, :hs]) for m in range(1, bits.shape[0]))
    return np.concatenate([np.ascontiguousarray(bits[0, :, :hs]).ravel(), np.ascontiguousarray(bits[:, :, hs:]).ravel()])


def unpack_dedup(flat, T, n, h, hs):
    """Inverse of pack_dedup: the shared block is broadcast to every rank."""
    out = np.empty((T, n, h), dtype=flat.dtype)
    out[:, :, :hs] = flat[:n * hs].reshape(1, n, hs)
    out[:, :, hs:] = flat[n * hs:].reshape(T, n, h - hs)
    return out
