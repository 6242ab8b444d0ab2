"""The floating-point parity bar, in one place.

bf16 outputs are compared with the oracle's UNROUNDED fp64 values:
    relative L2 error <= 5e-3 over the compared block, and per element
        |err| <= 2e-2                                   where |ref| < 8,
        |err| <= max(2e-2, half_ulp_bf16(ref) + 4e-3)   where |ref| >= 8.
The second line is the one exception to the plain bound, and it is forced by the output format: from
magnitude 8 on, neighbouring bf16 values are 2^-4 = 0.0625 or more apart, so the correctly rounded result
itself can be 0.03125 off and no bf16 output can promise 2e-2.  There the bound is the rounding of the
stored result plus 4e-3 for everything else.  Below 8 nothing is relaxed.
`assert_close` returns how many compared elements needed the exception (and the largest error among the
others), so that a test can report it.
fp32 workloads: max-abs <= 1e-4 and relative L2 <= 1e-5 (fp32 accumulation over K <= 512 terms).
"""
import numpy as np

TOL = {"bf16": (2e-2, 5e-3), "f32": (1e-4, 1e-5)}
BIG = 8.0          # from here on an absolute 2e-2 is not representable in bf16


def bf16_half_ulp(ref: np.ndarray) -> np.ndarray:
    """Half the spacing of bfloat16 values (8 significant bits) around ref, for normal magnitudes."""
    e = np.floor(np.log2(np.maximum(np.abs(ref), 2.0 ** -126)))
    return 2.0 ** (e - 8)


def bound_for(ref: np.ndarray, dtype: str) -> np.ndarray:
    ma, _ = TOL[dtype]
    bound = np.full(ref.shape, ma)
    if dtype == "bf16":
        big = np.abs(ref) >= BIG
        bound[big] = np.maximum(ma, bf16_half_ulp(ref[big]) + 4e-3)
    return bound


def assert_close(got, ref: np.ndarray, dtype: str = "bf16", what: str = ""):
    g = got.detach().double().cpu().numpy() if hasattr(got, "detach") else np.asarray(got, dtype=np.float64)
    stats = {"compared": int(ref.size), "over_plain": 0, "max_err_below_big": 0.0, "max_err": 0.0, "rel_l2": 0.0}
    if ref.size == 0:
        return stats
    assert g.shape == ref.shape, (g.shape, ref.shape)
    err = np.abs(g - ref)
    ma, rl = TOL[dtype]
    bound = bound_for(ref, dtype)
    rel = np.linalg.norm(g - ref) / max(np.linalg.norm(ref), 1e-30)
    worst = int(np.argmax(err / bound))
    assert (err <= bound).all() and rel <= rl, (
        f"{what}: worst |err| {err.flat[worst]:.3e} at |ref| {abs(ref.flat[worst]):.3e} "
        f"(bound {bound.flat[worst]:.3e}); {int((err > bound).sum())} of {ref.size} elements over their bound; "
        f"max-abs {err.max():.3e}, rel-L2 {rel:.3e} (<= {rl})")
    small = np.abs(ref) < BIG
    stats.update(over_plain=int((err > ma).sum()), max_err=float(err.max()), rel_l2=float(rel),
                 max_err_below_big=float(err[small].max()) if small.any() else 0.0)
    return stats
