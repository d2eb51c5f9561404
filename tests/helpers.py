"""Shared helpers of the GPU parity tests: error metric, upload, oracle calls on sampled sequences,
and the storage-rounding identity of bf16 outputs.

Tolerance: max |gpu - oracle| / rms(oracle) <= 1e-5 (fp32 inputs) / 2e-2 (bf16 inputs), on the bare
difference.  It is applied to results the GPU returns in fp32.  A result the GPU STORES as bf16
cannot be held to it by any implementation (an element 15 x the RMS large is stored no closer than
3 % of the RMS), so such results are checked in two exact steps instead: the same call with fp32
output meets the bare tolerance, and the bf16 result is that fp32 result rounded to nearest even,
bit for bit (`both_outputs`, `decode_both`, `assert_rne_bf16`)."""
import numpy as np

from paper_2507_01652_amd import workloads as wl

TOL = {"f32": 1e-5, "bf16": 2e-2}   # max |gpu - oracle| / rms(oracle), per input storage type


def rel_err(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if got.size == 0:
        return 0.0
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


def bf16_bits(t):
    """uint16 bit patterns of a torch bf16 tensor (host numpy array, logical order)."""
    import torch
    assert t.dtype == torch.bfloat16
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def assert_rne_bf16(t16, t32, what=""):
    """The bf16 result is the fp32 result rounded to nearest even, bit for bit (-0 and +0 alike)."""
    got = bf16_bits(t16)
    want = wl.f32_to_bf16_bits(t32.float().contiguous().cpu().numpy())
    same = (got == want) | (((got | want) & 0x7FFF) == 0)
    if not same.all():
        bad = np.argwhere(~same)
        i = tuple(bad[0])
        raise AssertionError(f"{what}: {len(bad)} of {got.size} bf16 outputs are not RNE of the fp32 output; first at {i}: "
                             f"bf16 bits {got[i]:#06x}, fp32 value {float(t32[i]):.9g} rounds to {want[i]:#06x}")


def both_outputs(fn, in_bf16, dtype_kw="out_dtype", state_kw="state_out", **kw):
    """Run fn(**kw) with fp32 output; with bf16 inputs run it again with bf16 output and require the bf16
    result(s) to be the rounded fp32 result(s) and the final state to be the same.  Returns what the fp32
    call returned (compare THAT with the oracle at the bare tolerance).  fn returns a tensor or a tuple of
    tensors; fp32 members of a tuple (dgamma, dweight) must be equal in both runs."""
    import torch
    r32 = fn(**{**kw, dtype_kw: torch.float32})
    torch.cuda.synchronize()
    if not in_bf16:
        return r32
    st = kw.get(state_kw)
    st32 = None if st is None else st.clone()
    r16 = fn(**{**kw, dtype_kw: torch.bfloat16})
    torch.cuda.synchronize()
    a32 = r32 if isinstance(r32, (tuple, list)) else (r32,)
    a16 = r16 if isinstance(r16, (tuple, list)) else (r16,)
    for i, (x16, x32) in enumerate(zip(a16, a32)):
        if x16 is None:
            continue
        if x16.dtype == torch.bfloat16:
            assert_rne_bf16(x16, x32, f"{getattr(fn, '__name__', 'call')} output {i}")
        else:
            assert torch.equal(x16, x32), f"fp32 output {i} differs between the two runs"
    if st is not None:
        assert torch.equal(st, st32), "final state differs between the fp32-output and the bf16-output run"
    return r32


def decode_both(step, state, in_bf16):
    """One decode step, state updated in place: step(state, out_dtype) -> o.  With bf16 inputs the step is run
    on a copy of the incoming state with bf16 output as well: same new state, o rounded.  Returns the fp32 o."""
    import torch
    before = state.clone() if in_bf16 else None
    o32 = step(state, torch.float32)
    if in_bf16:
        o16 = step(before, torch.bfloat16)
        torch.cuda.synchronize()
        assert_rne_bf16(o16, o32, "decode step")
        assert torch.equal(before, state), "new state differs between the fp32-output and the bf16-output run"
    return o32
