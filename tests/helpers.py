"""Shared helpers of the GPU parity tests: error metric, upload, oracle calls on sampled sequences."""
import numpy as np

TOL = {"f32": 1e-5, "bf16": 2e-2}   # max |gpu - oracle| / rms(oracle), per input storage type


def rel_err(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rms = np.sqrt(np.mean(ref * ref))
    if rms == 0.0:
        return float(np.max(np.abs(got - ref)))
    return float(np.max(np.abs(got - ref)) / rms)


def sample_pairs(B, Hh, count, seed):
    """`count` distinct (b, h) pairs, always including the first and the last sequence."""
    rng = np.random.default_rng(seed)
    total = B * Hh
    count = min(count, total)
    idx = {0, total - 1}
    while len(idx) < count:
        idx.add(int(rng.integers(total)))
    return [(i // Hh, i % Hh) for i in sorted(idx)]


def gather_pairs(x, pairs):
    """[B, n, Hh, d] -> [1, n, len(pairs), d]: the sampled sequences laid out as heads."""
    return np.stack([x[b, :, h, :] for b, h in pairs], axis=1)[None]


def bf16_half_ulp(x):
    """Half the spacing of bf16 values (8 significant bits) at |x|: the largest error that
    round-to-nearest storage of a value landing on x can carry; between 2^-9 and 2^-8 of |x|."""
    ax = np.abs(np.asarray(x, dtype=np.float64))
    e = np.floor(np.log2(np.where(ax > 0, ax, 1.0)))
    return np.where(ax > 0, 2.0 ** (e - 8.0), 0.0)


def parity_err(got, ref, out_bf16):
    """max |gpu - oracle| / rms(oracle).  When the GPU result was STORED as bf16, the storage
    rounding of that one element (half a bf16 spacing at its magnitude, whatever computed it) is
    taken off first: the tolerance is on the computation, and an output element 15 x the RMS
    cannot be stored in bf16 more closely than 3 % of the RMS by any implementation."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if got.size == 0:
        return 0.0
    diff = np.abs(got - ref)
    if out_bf16:
        diff = np.maximum(diff - bf16_half_ulp(got), 0.0)
    rms = np.sqrt(np.mean(ref * ref))
    return float(diff.max() / rms) if rms > 0 else float(diff.max())
