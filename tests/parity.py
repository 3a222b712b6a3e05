"""Error measures and oracle adapters shared by the GPU parity tests."""
import numpy as np
import torch

# Tolerances on max|x - ref| / max|ref| per output tensor.
# (fp16 is not one of the benchmark's dtypes; its bound is the bf16 one scaled by the ratio of the unit
# roundoffs, 2^-11 against 2^-8.)
TOL = {torch.float32: 1e-5, torch.bfloat16: 2e-2, torch.float16: 2.5e-3}
# rms(x - ref) / rms(ref): what bf16 operand rounding (2^-9 per element) is expected to stay under.
RMS_TOL = {torch.float32: 5e-6, torch.bfloat16: 1e-2, torch.float16: 1.25e-3}


def to64(t):
    """Exact up-cast of a torch tensor (bf16 / fp32, any device) to a numpy float64 array."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def max_rel(x, ref):
    den = float(np.max(np.abs(ref))) if ref.size else 0.0
    if ref.size == 0:
        return 0.0
    if den == 0.0:
        return float(np.max(np.abs(x)))
    return float(np.max(np.abs(x - ref))) / den


def rms_rel(x, ref):
    if ref.size == 0:
        return 0.0
    den = float(np.sqrt(np.mean(ref * ref)))
    num = float(np.sqrt(np.mean((x - ref) ** 2)))
    return num / den if den > 0 else num


def assert_close(name, got, ref, dtype):
    """got: torch tensor from the GPU; ref: float64 numpy oracle values."""
    x = to64(got)
    assert x.shape == ref.shape, (name, x.shape, ref.shape)
    assert np.all(np.isfinite(x)), "%s: non-finite values" % name
    m, r = max_rel(x, ref), rms_rel(x, ref)
    assert m <= TOL[dtype], "%s: max rel err %.3e > %.1e (rms rel %.3e)" % (name, m, TOL[dtype], r)
    assert r <= RMS_TOL[dtype], "%s: rms rel err %.3e > %.1e" % (name, r, RMS_TOL[dtype])
    # element by element: the same tolerance against each element's own magnitude plus a floor of a quarter of
    # the tensor's largest magnitude (small elements of a signed sum have no relative accuracy of their own;
    # the floor makes their bound four times tighter than the max-norm bound above)
    if ref.size:
        floor = 0.25 * float(np.max(np.abs(ref)))
        e = float(np.max(np.abs(x - ref) / (np.abs(ref) + floor))) if floor > 0 else float(np.max(np.abs(x)))
        assert e <= TOL[dtype], "%s: element-wise err %.3e > %.1e" % (name, e, TOL[dtype])
    return m, r
