"""Comparison helpers for the parity tests (HIP path vs CPU oracle).  Not a test module.

Tolerances (bf16 output, fp32 accumulation):
  O    |dO| <= 1e-2 * max(1, |O_ref|) element-wise: max-abs 1e-2 wherever |O_ref| <= 1; above that the bf16
       output format alone rounds by up to 2^-9 * |O| (0.0156 at |O| = 4, reached by rows that see only a
       few N(0,1) value rows), so the bound scales with the magnitude.  AND per (row, head)
       max|dO| <= (1 + r) * 2^-8 * max|O_ref| + 1e-5 and cosine >= 0.999 (these keep the test meaningful for
       long KV, where |O| ~ 1/sqrt(n) is tiny and an all-zero output would pass the absolute bound), with r the
       number of bf16 roundings between the fp32 arithmetic and the compared value: 1 for a kernel's own output
       (2^-8 for that rounding, another 2^-8 for the bf16 probabilities of the second product), 2 for a merge
       of bf16 partials (each partial was rounded once already);
  LSE  |dLSE| <= 1e-4 * max(1, |LSE_ref|), and -inf must match exactly.
"""
import numpy as np

O_ABS_TOL = 1e-2
O_REL_UNIT = 2.0 ** -8
LSE_REL_TOL = 1e-4


def check_o_lse(O_gpu, LSE_gpu, O_ref, LSE_ref, what="", roundings=1):
    """O_* [n, D], LSE_* [n]; gpu values as float64 arrays; roundings: see the module docstring."""
    O_gpu = np.asarray(O_gpu, np.float64); LSE_gpu = np.asarray(LSE_gpu, np.float64)
    assert O_gpu.shape == O_ref.shape and LSE_gpu.shape == LSE_ref.shape, what
    assert not np.isnan(O_gpu).any() and not np.isnan(LSE_gpu).any(), f"{what}: NaN in GPU output"
    empty = np.isneginf(LSE_ref)
    assert np.array_equal(np.isneginf(LSE_gpu), empty), f"{what}: -inf pattern of LSE differs"
    assert (O_gpu[empty] == 0).all(), f"{what}: rows with no visible key must be zero"
    fin = ~empty
    if not fin.any():
        return dict(o_abs=0.0, lse_err=0.0)
    dl = np.abs(LSE_gpu[fin] - LSE_ref[fin])
    lim = LSE_REL_TOL * np.maximum(1.0, np.abs(LSE_ref[fin]))
    assert (dl <= lim).all(), f"{what}: LSE error {dl.max():.3e} (worst ratio {np.max(dl / lim):.2f})"
    dO = np.abs(O_gpu[fin] - O_ref[fin])
    o_abs = dO.max()
    worst = np.max(dO / np.maximum(1.0, np.abs(O_ref[fin])))
    assert worst <= O_ABS_TOL, f"{what}: O error {worst:.3e} (in units of max(1, |O_ref|)); max-abs {o_abs:.3e}"
    row_ref = np.abs(O_ref[fin]).max(axis=1)
    row_err = dO.max(axis=1)
    bad = row_err > (1 + roundings) * O_REL_UNIT * row_ref + 1e-5
    assert not bad.any(), f"{what}: relative O error, worst {np.max(row_err / (row_ref + 1e-30)):.3e}"
    num = (O_gpu[fin] * O_ref[fin]).sum(1)
    den = np.linalg.norm(O_gpu[fin], axis=1) * np.linalg.norm(O_ref[fin], axis=1)
    ok = den > 0
    assert (num[ok] / den[ok] >= 0.999).all(), f"{what}: cosine similarity {np.min(num[ok] / den[ok]):.5f}"
    return dict(o_abs=float(o_abs), lse_err=float(dl.max()))


def sample_rows(rng, lo, hi, n_random, edges=(16, 32, 64, 128, 256)):
    """Row indices in [lo, hi): first/last, tile edges +-1, plus random rows."""
    rows = {lo, hi - 1}
    for e in edges:
        for base in range(lo, hi, e):
            for d in (-1, 0, 1):
                r = base + d
                if lo <= r < hi:
                    rows.add(r)
            if len(rows) > 64:
                break
    rows = sorted(rows)
    if len(rows) > 48:
        keep = rng.choice(len(rows), 48, replace=False)
        rows = sorted({rows[i] for i in keep} | {lo, hi - 1})
    extra = rng.integers(lo, hi, n_random)
    return np.unique(np.concatenate([np.asarray(rows, np.int64), extra.astype(np.int64)]))
