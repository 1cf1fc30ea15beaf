"""Comparison helpers for the parity tests (HIP path vs CPU oracle).  Not a test module.

Tolerances (bf16 output, fp32 accumulation):
  O    |dO| <= max(1e-2, 2^-8 * |O_ref|) element-wise, plus 2^-9 * |O_ref| from |O_ref| = 4 up.  The stated max-abs
       1e-2 holds wherever |O_ref| <= 2.56.  Above that the bf16 output format alone rounds by up to half a unit in
       the last place, at most 2^-8 * |O|; but just above a power of two it is exactly that (0.015625 for a value a
       little over 4.0, which rows that see only a few N(0,1) value rows reach), so there the format's bound leaves
       nothing for the error the value carries BEFORE it is rounded: the probabilities are rounded to bf16 for the
       second product, half a unit each, 2^-9 relative.  That term is added from 4.0 up; below, where the format
       leaves room (half a unit is 0.0078 in [2, 4)), it is not.  (Without it, an element whose exact value sits
       just above 4.0156, the midpoint of two bf16 values, and that was 4e-4 off before the rounding, fails at
       1.024 x the bound: seen once.)  How many compared elements fell into the scaled
       region is returned (`o_scaled`) and printed.  AND per (row, head)
       max|dO| <= 2^-7 * max|O_ref| + 1e-5 and cosine >= 0.999 (these keep the test meaningful for long KV,
       where |O| ~ 1/sqrt(n) is tiny and an all-zero output would pass the absolute bound): 2^-8 for the one
       rounding of the output to bf16, another 2^-8 for the bf16 probabilities of the second product.  Every
       compared value is rounded to bf16 once: a kernel's own output, a merge of fp32 partials against attention
       over the union of the shards, or a merge of bf16 partials against the oracle's merge of those very arrays;
  LSE  |dLSE| <= 1e-4 * max(1, |LSE_ref|), and -inf must match exactly.
"""
import numpy as np

O_ABS_TOL = 1e-2
O_REL_UNIT = 2.0 ** -8             # one rounding to bf16, worst case relative to the value
O_PROB_UNIT = 2.0 ** -9            # the probabilities' rounding to bf16, counted from |O_ref| = 4 up
LSE_REL_TOL = 1e-4


def check_o_lse(O_gpu, LSE_gpu, O_ref, LSE_ref, what=""):
    """O_* [n, D], LSE_* [n]; gpu values as float64 arrays."""
    O_gpu = np.asarray(O_gpu, np.float64); LSE_gpu = np.asarray(LSE_gpu, np.float64)
    assert O_gpu.shape == O_ref.shape and LSE_gpu.shape == LSE_ref.shape, what
    assert not np.isnan(O_gpu).any() and not np.isnan(LSE_gpu).any(), f"{what}: NaN in GPU output"
    empty = np.isneginf(LSE_ref)
    assert np.array_equal(np.isneginf(LSE_gpu), empty), f"{what}: -inf pattern of LSE differs"
    assert (O_gpu[empty] == 0).all(), f"{what}: rows with no visible key must be zero"
    fin = ~empty
    if not fin.any():
        return dict(o_abs=0.0, lse_err=0.0, o_scaled=0, o_compared=0)
    dl = np.abs(LSE_gpu[fin] - LSE_ref[fin])
    lim = LSE_REL_TOL * np.maximum(1.0, np.abs(LSE_ref[fin]))
    assert (dl <= lim).all(), f"{what}: LSE error {dl.max():.3e} (worst ratio {np.max(dl / lim):.2f})"
    dO = np.abs(O_gpu[fin] - O_ref[fin])
    o_abs = dO.max()
    a_ref = np.abs(O_ref[fin])
    o_lim = np.maximum(O_ABS_TOL, O_REL_UNIT * a_ref) + np.where(a_ref >= 4.0, O_PROB_UNIT * a_ref, 0.0)
    worst = np.max(dO / o_lim)
    assert worst <= 1.0, f"{what}: O error {worst:.3f} x the bound max(1e-2, 2^-8 |O_ref|) (+ 2^-9 |O_ref| from 4 up); max-abs {o_abs:.3e}"
    o_scaled = int((o_lim > O_ABS_TOL).sum())
    row_ref = np.abs(O_ref[fin]).max(axis=1)
    row_err = dO.max(axis=1)
    bad = row_err > 2 * O_REL_UNIT * row_ref + 1e-5
    assert not bad.any(), f"{what}: relative O error, worst {np.max(row_err / (row_ref + 1e-30)):.3e}"
    num = (O_gpu[fin] * O_ref[fin]).sum(1)
    den = np.linalg.norm(O_gpu[fin], axis=1) * np.linalg.norm(O_ref[fin], axis=1)
    ok = den > 0
    assert (num[ok] / den[ok] >= 0.999).all(), f"{what}: cosine similarity {np.min(num[ok] / den[ok]):.5f}"
    st = dict(o_abs=float(o_abs), lse_err=float(dl.max()), o_scaled=o_scaled, o_compared=int(dO.size))
    print(f"[check] {what}: max|dO| {st['o_abs']:.2e} over {st['o_compared']} elements ({o_scaled} of them above |O_ref| = 2.56, "
          f"bound 2^-8 |O_ref| there, + 2^-9 |O_ref| from 4 up), max|dLSE| {st['lse_err']:.2e} over {int(fin.sum())} rows", flush=True)
    return st
