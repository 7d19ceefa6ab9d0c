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


WORST = {}  # what -> (max-norm ratio, worst per-row ratio), both in units of rtol; printed by the tests


def assert_close_rows(got, ref, rtol, width, what):
    """max-norm error <= rtol * max-norm of the oracle, and per-row (per-slice) relative L2
    error <= rtol for every row whose oracle norm is not negligible (above 1e-3 of the largest
    row norm: a row that is small because its terms cancel has an absolute, not a relative, error
    bound, and that bound is the max-norm test).  Rows the oracle leaves at 0 must be exactly 0."""
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
    worst = 0.0
    if sig.any():
        worst = (en[sig] / rn[sig]).max()
        assert worst <= rtol, "%s: worst row-relative L2 error %.3e" % (what, worst)
    WORST[what] = (err / (rtol * scale) if scale > 0 else 0.0, worst / rtol)
    zero = rn == 0.0
    assert np.all(got[zero] == 0.0), "%s: rows the oracle leaves at 0 must be exactly 0" % what


def report_worst(prefix=""):
    """One line per compared tensor: the observed errors as fractions of the tolerance."""
    for what, (a, b) in sorted(WORST.items()):
        print("  tol-use %s%s: max-norm %.3f, per-row L2 %.3f" % (prefix, what, a, b), flush=True)
    WORST.clear()


def slice_view(shape, k, flat):
    """Core gradient k as [n_k][everything else] so that each row is one slice."""
    a = np.asarray(flat).reshape(shape.r[k], shape.n[k], shape.d[k] * shape.r[k + 1])
    return np.ascontiguousarray(a.transpose(1, 0, 2)).reshape(shape.n[k], -1)


def assert_grads_close(shape, got, ref, rtol=GRAD_RTOL, what="dG"):
    for k in range(3):
        g = got[k].detach().cpu().numpy() if torch.is_tensor(got[k]) else got[k]
        w = shape.r[k] * shape.d[k] * shape.r[k + 1]
        assert_close_rows(slice_view(shape, k, g), slice_view(shape, k, ref[k]), rtol, w, "%s%d" % (what, k + 1))


def assert_plan_equals_oracle(ora, shape, plan, idx, off, remap=None):
    """Every index array of the GPU plan, bit for bit, against the integer oracle (stable sort by
    row + unique) and against numpy's stable argsort / searchsorted for the groupings."""
    ref = ora.reorder_plan(shape, idx, off, remap=remap)
    got = plan.arrays()
    nv = ref["num_valid"]
    assert got["num_valid"] == nv and got["U_r"] == len(ref["uniq_row"]) and got["U_p"] == len(ref["uniq_pref"])
    for key in ("perm", "sorted_row", "bag_of_sorted"):
        assert np.array_equal(got[key][:nv], ref[key]), key
    for key in ("uniq_row", "row_seg", "lookup2row", "uniq_pref", "pref_seg", "row2pref"):
        assert np.array_equal(got[key], ref[key]), key
    i3 = ref["uniq_row"] % shape.n[2]
    assert np.array_equal(got["rows_by_i3"], np.argsort(i3, kind="stable"))
    assert np.array_equal(got["i3_of_sorted"], np.sort(i3))
    assert np.array_equal(got["i3_seg"], np.searchsorted(np.sort(i3), np.arange(shape.n[2] + 1)))
    i2 = ref["uniq_pref"] % shape.n[1]
    assert np.array_equal(got["prefs_by_i2"], np.argsort(i2, kind="stable"))
    assert np.array_equal(got["i2_seg"], np.searchsorted(np.sort(i2), np.arange(shape.n[1] + 1)))
    i1 = ref["uniq_pref"] // shape.n[1]
    assert np.array_equal(got["i1_seg"], np.searchsorted(i1, np.arange(shape.n[0] + 1)))
    return got
