"""Shared helpers of the GPU parity tests: tolerances (stated once, here) and comparisons.

Tolerances
----------
fp32 path      : max |gpu - oracle| / max |oracle| <= 1e-5 per output tensor (norm-wise maximum).
16-bit path    : partial / merged outputs: max abs error <= 2e-2; log-sum-exp: max abs error <= 1e-3.
scramble, 16-bit storage: the kernel accumulates the d exact products of a row in fp32 and rounds once
                 (RNE) to the storage type.  Against round(oracle) this allows one storage ulp where the
                 fp32 sum lands on the other side of a rounding boundary, plus the fp32 accumulation error,
                 bounded by d * 2^-24 * sum_k |x_k Phi_kj| <= 1e-5 * sum_k |x_k Phi_kj| for d <= 128:
                     |gpu - round(oracle)| <= ulp_storage(oracle) + 2e-5 * sum_k |x_k| |Phi_kj|
                 and at least 97 % of the elements must match bit for bit.
                 One flat output bound for every 16-bit attention call, the Inquirer's local attention on
                 plaintext V (outlier channels not spread by Phi, |v| up to ~80) included.
Index work     : bit-exact.
"""
import numpy as np
import torch

TOL_F32_REL = 1e-5
TOL_16_OUT_ABS = 2e-2
TOL_16_LSE_ABS = 1e-3

_MANT = {torch.bfloat16: 7, torch.float16: 10}


def f64(t):
    return t.detach().cpu().double().numpy() if hasattr(t, "detach") else np.asarray(t, dtype=np.float64)


def rel_normwise(got, ref):
    got, ref = f64(got), np.asarray(ref, dtype=np.float64)
    fin = np.isfinite(ref)
    assert np.array_equal(np.isfinite(got), fin), "finite / infinite pattern differs"
    if not fin.any():
        return 0.0
    assert np.array_equal(got[~fin], ref[~fin])
    den = np.abs(ref[fin]).max()
    return float(np.abs(got[fin] - ref[fin]).max() / max(den, 1e-30))


def max_abs(got, ref):
    got, ref = f64(got), np.asarray(ref, dtype=np.float64)
    fin = np.isfinite(ref)
    assert np.array_equal(np.isfinite(got), fin), "finite / infinite pattern differs"
    assert np.array_equal(got[~fin], ref[~fin])
    return float(np.abs(got[fin] - ref[fin]).max()) if fin.any() else 0.0


def check_attn(got_O, got_lse, ref_O, ref_lse, dtype, what="", report=False):
    """Returns the observed (output, lse) errors; report=True also prints them (pytest -s / a failing test shows it)."""
    if dtype == torch.float32:
        eo, el = rel_normwise(got_O, ref_O), rel_normwise(got_lse, ref_lse)
        if report:
            print(f"{what}: observed O rel err {eo:.3e}, lse rel err {el:.3e} (bound {TOL_F32_REL:.0e})")
        assert eo <= TOL_F32_REL, f"{what}: O rel err {eo:.3e}"
        assert el <= TOL_F32_REL, f"{what}: lse rel err {el:.3e}"
    else:
        eo, el = max_abs(got_O, ref_O), max_abs(got_lse, ref_lse)
        if report:
            print(f"{what}: observed O abs err {eo:.3e} (bound {TOL_16_OUT_ABS:.0e}), lse abs err {el:.3e} "
                  f"(bound {TOL_16_LSE_ABS:.0e})")
        assert eo <= TOL_16_OUT_ABS, f"{what}: O abs err {eo:.3e} > {TOL_16_OUT_ABS:.0e}"
        assert el <= TOL_16_LSE_ABS, f"{what}: lse abs err {el:.3e}"
    return eo, el


def storage_ulp(ref64, dtype):
    mant = _MANT[dtype]
    a = np.abs(ref64)
    e = np.floor(np.log2(np.maximum(a, 1e-300)))
    if dtype == torch.float16:
        e = np.maximum(e, -14)
    else:
        e = np.maximum(e, -126)
    return np.exp2(e - mant)


def check_scramble(got, ref64, X, Phi, perm, G, dtype, what=""):
    """got: device/CPU tensor in storage dtype; ref64: oracle result (fp64); X, Phi the inputs as consumed."""
    got64 = f64(got)
    if dtype == torch.float32:
        e = rel_normwise(got64, ref64)
        assert e <= TOL_F32_REL, f"{what}: rel err {e:.3e}"
        return e
    rounded = torch.from_numpy(ref64).to(dtype).double().numpy()
    X64, P64 = np.abs(f64(X)), np.abs(f64(Phi))
    B, H, L, d = X64.shape
    if perm is not None:
        p = np.asarray(perm.cpu() if hasattr(perm, "cpu") else perm)
        if p.ndim == 1:
            p = np.broadcast_to(p, (B, L))
        elif p.shape[0] == 1:
            p = np.broadcast_to(p[0], (B, L))
        X64 = np.stack([X64[b][:, p[b]] for b in range(B)])
    mag = np.einsum("bhlk,hkj->bhlj", X64, np.repeat(P64, G, axis=0))
    tol = storage_ulp(rounded, dtype) + 2e-5 * mag
    diff = np.abs(got64 - rounded)
    worst = float((diff / tol).max())
    assert worst <= 1.0, f"{what}: |gpu - round(oracle)| exceeds ulp + fp32 accumulation bound by x{worst:.2f}"
    exact = float((diff == 0).mean())
    assert exact >= 0.97, f"{what}: only {exact:.4f} of elements bit-identical to round(oracle)"
    return exact
