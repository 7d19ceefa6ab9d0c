"""Helpers of the GPU parity tests: marshalling to the C-ABI binding and the comparison metric."""
import numpy as np
import torch

import paper_2507_14668_amd as tt

FWD_RTOL = 1e-5   # forward outputs (fp32), stated by the target
GRAD_RTOL = 1e-4  # core gradients and updated cores (fp32), stated by the target


def to_dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def gpu_table(shape, cores):
    return tt.Table.from_numpy(shape, [np.asarray(c, dtype=np.float32) for c in cores])


def assert_close_rows(got, ref, rtol, width, what):
    """max-norm error <= rtol * max-norm of the oracle, and per-row (per-slice) relative L2
    error <= rtol for every row whose oracle norm is not negligible."""
    got = np.asarray(got, dtype=np.float64).reshape(-1, width)
    ref = np.asarray(ref, dtype=np.float64).reshape(-1, width)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), what
    scale = np.abs(ref).max() if ref.size else 0.0
    err = np.abs(got - ref).max() if ref.size else 0.0
    assert err <= rtol * scale + 1e-30, "%s: max err %.3e vs scale %.3e" % (what, err, scale)
    rn = np.linalg.norm(ref, axis=1)
    en = np.linalg.norm(got - ref, axis=1)
    sig = rn > 1e-3 * (rn.max() if rn.size else 0.0) + 1e-30
    if sig.any():
        worst = (en[sig] / rn[sig]).max()
        assert worst <= 4 * rtol, "%s: worst row-relative L2 error %.3e" % (what, worst)
    zero = rn == 0.0
    assert np.all(got[zero] == 0.0), "%s: rows the oracle leaves at 0 must be exactly 0" % what


def slice_view(shape, k, flat):
    """Core gradient k as [n_k][everything else] so that each row is one slice."""
    a = np.asarray(flat).reshape(shape.r[k], shape.n[k], shape.d[k] * shape.r[k + 1])
    return np.ascontiguousarray(a.transpose(1, 0, 2)).reshape(shape.n[k], -1)


def assert_grads_close(shape, got, ref, rtol=GRAD_RTOL, what="dG"):
    for k in range(3):
        g = got[k].detach().cpu().numpy() if torch.is_tensor(got[k]) else got[k]
        w = shape.r[k] * shape.d[k] * shape.r[k + 1]
        assert_close_rows(slice_view(shape, k, g), slice_view(shape, k, ref[k]), rtol, w, "%s%d" % (what, k + 1))
