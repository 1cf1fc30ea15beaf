"""Comparison helpers for the parity tests (HIP path vs CPU oracle).  Not a test module.

Tolerances (bf16 output, fp32 accumulation):
  O    |dO| <= 1e-2 element-wise, the stated max-abs, wherever |O_ref| <= 2.56; above that the bf16 output format
       alone rounds by up to half a unit in the last place, which is 2^-8 * |O| for a value just above a power of
       two (0.0156 at |O| = 4.0, reached by rows that see only a few N(0,1) value rows), and the value that gets
       rounded already carries the rounding of the probabilities to bf16 before the second product, half a unit
       each, 2^-9 relative: there the bound is (2^-8 + 2^-9) * |O_ref|.  (With 2^-8 alone, an element whose exact
       value sits just above 4 and whose rounding goes the wrong way fails by the few 1e-4 of error it had before
       the rounding: seen once, at 1.024 x that bound.)  How many compared elements fell into the scaled
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
O_ELEM_UNIT = 1.5 * 2.0 ** -8      # element-wise: the output's rounding plus the probabilities'
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
    o_lim = np.where(a_ref <= O_ABS_TOL / O_REL_UNIT, O_ABS_TOL, O_ELEM_UNIT * a_ref)
    worst = np.max(dO / o_lim)
    assert worst <= 1.0, f"{what}: O error {worst:.3f} x the bound (1e-2, or 1.5 * 2^-8 |O_ref| above |O_ref| = 2.56); max-abs {o_abs:.3e}"
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
          f"bound 1.5 * 2^-8 |O_ref| there), max|dLSE| {st['lse_err']:.2e} over {int(fin.sum())} rows", flush=True)
    return st
