"""The attention tolerance, in one place for every GPU test.

fp32 path: 1e-4 absolute (the spec bar).

bf16 path: the spec bar is 2e-2 absolute.  It is asserted as it stands on every output
element whose attended magnitude  mag = sum_i a_i |v_i|  (the oracle's attention applied to |V|)
is at most 4: there the bf16 storage of the output (half a unit in the last place, at most
2^-9 |o| <= 2^-9 mag < 8e-3) cannot be what decides.  Above that magnitude the output's own bf16
spacing approaches and passes 2e-2 (spacing 3.1e-2 from |o| = 4, 6.3e-2 from |o| = 8), and
the bound is 2e-2 + 2^-8 mag: half a unit of output rounding plus as much again for the softmax
weights, which enter the second matrix product rounded to bf16.

Every check also records how much of that slack was used: how many elements were above the flat
2e-2 at all, how many of those were still above 2e-2 + the output's own bf16 half-spacing
2^-9 |ref| (i.e. needed part of the weight-rounding share), and the largest error and magnitude.
The records are printed in the terminal summary of the test run (see conftest.py).
"""
import numpy as np

FLAT_BF16 = 2e-2
FLAT_F32 = 1e-4
MAG_FLAT_LIMIT = 4.0

REPORT = []     # one line per check


def check_attention(got, ref, mag, dtype, label):
    """Asserts the tolerance described in the module docstring; returns the record that was logged."""
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    err = np.abs(got - ref)
    assert np.all(np.isfinite(got)), f"{label}: non-finite output"
    if dtype == "f32":
        worst = np.unravel_index(np.argmax(err), err.shape)
        assert np.all(err <= FLAT_F32), f"{label}: fp32 attention error {err[worst]} at {worst}"
        rec = dict(label=label, elements=int(err.size), max_err=float(err.max()), over_flat=0, over_flat_plus_store=0,
                   max_mag=None)
        REPORT.append(f"{label}: fp32, {err.size} elements, max err {err.max():.2e} (bar {FLAT_F32})")
        return rec
    mag = np.abs(ref) if mag is None else np.asarray(mag, np.float64)
    low = mag <= MAG_FLAT_LIMIT
    tol = np.where(low, FLAT_BF16, FLAT_BF16 + mag * 2.0 ** -8)
    excess = err - tol
    worst = np.unravel_index(np.argmax(excess), err.shape)
    assert np.all(excess <= 0), (f"{label}: attention error {err[worst]} at {worst} (got {got[worst]}, ref {ref[worst]}, "
                                 f"attended magnitude {mag[worst]}, bound {tol[worst]})")
    over_flat = err > FLAT_BF16
    over_store = err > FLAT_BF16 + np.abs(ref) * 2.0 ** -9
    rec = dict(label=label, elements=int(err.size), low_mag_elements=int(low.sum()), max_err=float(err.max()),
               max_err_low_mag=float(err[low].max()) if low.any() else 0.0,
               over_flat=int(over_flat.sum()), over_flat_plus_store=int(over_store.sum()), max_mag=float(mag.max()),
               max_err_over_flat_at_mag=float(mag[over_flat].min()) if over_flat.any() else None)
    REPORT.append(f"{label}: bf16, {err.size} elements ({int(low.sum())} with magnitude <= {MAG_FLAT_LIMIT}: flat 2e-2 asserted, "
                  f"max err there {rec['max_err_low_mag']:.2e}); max err {err.max():.2e}, max magnitude {mag.max():.2f}; "
                  f"{rec['over_flat']} elements above the flat 2e-2"
                  + (f" (smallest magnitude among them {rec['max_err_over_flat_at_mag']:.1f})" if over_flat.any() else "")
                  + f", {rec['over_flat_plus_store']} above 2e-2 + output half-spacing")
    return rec


def check_topk_band(idx, score_ref, k, rtol=2e-5):
    """idx is a valid top-k of scores that agree with score_ref to rtol: everything clearly above
    the k-th reference score is in, everything clearly below is out, indices ascending/unique."""
    idx = np.asarray(idx)
    assert len(idx) == k
    if k == 0:
        return
    assert np.all(np.diff(idx) > 0) and idx[0] >= 0 and idx[-1] < len(score_ref)
    thr = np.sort(score_ref)[::-1][k - 1]
    chosen = np.zeros(len(score_ref), bool)
    chosen[idx] = True
    assert np.all(chosen[score_ref > thr * (1 + rtol) + 1e-30]), "a clearly better candidate was left out"
    assert not np.any(chosen[score_ref < thr * (1 - rtol) - 1e-30]), "a clearly worse candidate was taken"
