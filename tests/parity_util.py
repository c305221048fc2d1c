"""Helpers shared by the GPU parity tests: tolerances, error metric, sampling."""
import numpy as np

# Tolerances stated for the method's target: maximum error relative to the largest reference
# magnitude of the tensor (element-wise relative error is unbounded where sums cancel).
TOL = {"f32": 1e-5, "bf16": 2e-2}


def max_rel_err(y, ref):
    y = np.asarray(y, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    scale = np.abs(ref).max()
    if scale == 0:
        return float(np.abs(y).max())
    return float(np.abs(y - ref).max() / scale)


def pass_rate(y, ref, tol):
    """Share of the elements with |y - ref| <= tol * |ref| + tol * rms(ref): the element-wise reading of the
    stated tolerance (the rms term keeps sums that cancel to almost nothing from deciding it)."""
    y = np.asarray(y, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 1.0
    rms = float(np.sqrt(np.mean(ref * ref)))
    return float(np.mean(np.abs(y - ref) <= tol * np.abs(ref) + tol * rms))


# one line per comparison, printed by conftest.py at the end of the run: both readings of the tolerance
PARITY_LOG = []


def assert_close(y, ref, dtype, what=""):
    assert np.all(np.isfinite(np.asarray(y, dtype=np.float64))), f"{what}: non-finite output"
    err = max_rel_err(y, ref)
    rate = pass_rate(y, ref, TOL[dtype])
    PARITY_LOG.append(f"{what or 'case'} [{dtype}, {np.asarray(ref).size} outputs]: max|y - ref| / max|ref| = {err:.3e} "
                      f"(limit {TOL[dtype]:.0e}), element-wise pass rate = {rate:.6f}")
    assert err <= TOL[dtype], f"{what}: max error / max|ref| = {err:.3e} > {TOL[dtype]:.1e}"
    assert rate >= 0.9999, f"{what}: only {rate:.6f} of the outputs are within the element-wise tolerance"
    return err


def sample_linear(M, cout, cin, p, count, seed):
    """(rows, cols) of outputs to check at full size: random ones plus the first / last rows and
    columns and every column whose weight row touches a tile (and alpha) boundary."""
    rng = np.random.default_rng(seed)
    rows = [rng.integers(0, M, size=count)]
    cols = [rng.integers(0, cout, size=count)]
    edge_cols = {0, cout - 1}
    n = cin * cout
    for f in range(p, n, p):          # tile boundaries in the flattened weight
        o = f // cin
        for d in (-1, 0, 1):
            if 0 <= o + d < cout:
                edge_cols.add(o + d)
    edge_cols = np.array(sorted(edge_cols), dtype=np.int64)
    edge_rows = np.array(sorted({0, M - 1, M // 2, min(M - 1, 31), min(M - 1, 32)}), dtype=np.int64)
    rr, cc = np.meshgrid(edge_rows, edge_cols, indexing="ij")
    rows.append(rr.reshape(-1))
    cols.append(cc.reshape(-1))
    rr, cc = np.meshgrid(edge_rows, rng.integers(0, cout, size=64), indexing="ij")
    rows.append(rr.reshape(-1))
    cols.append(cc.reshape(-1))
    return np.concatenate(rows).astype(np.int64), np.concatenate(cols).astype(np.int64)
