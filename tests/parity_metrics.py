"""Error measures for the gradients of the output layer that can see the softmax half of D.

The stated parity bar is max|got - ref| <= tol * max|ref| over a whole tensor.  For dW (and
nearly for dH) that maximum is set by the one-hot half of D = (softmax - G) * scale: a vocabulary
row that carries labels receives -scale * H_i terms of order |H|/N, while the softmax half of a
row is of order |H| / (V sqrt(N)).  At large V a kernel that dropped the softmax half entirely
would still pass.  The measures below remove the one-hot half (which is exact data movement in
the definition: rows of W and of H) and normalise what is left by its own maximum:

  * dH_i + scale * W[g_i]            = scale * sum_j softmax_ij W_j        (section 4.2, dX with G taken out)
  * rows j of dW that carry no label = scale * sum_i softmax_ij H_i        (section 4.2, dW with G_j = 0)
  * D element by element             = (softmax - G) * scale, relative to |D_ij|

NumPy only, no method arithmetic beyond adding the one-hot rows back; used by the GPU parity
tests and by a CPU test that plants mistakes in the oracle's D to show which measure sees them.
"""
from __future__ import annotations

import numpy as np


def rel_max_err(got: np.ndarray, ref: np.ndarray) -> float:
    """The stated bar's measure: max-abs error over max-abs of the reference."""
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-300))


def dH_softmax_part_err(dH_got: np.ndarray, dH_ref: np.ndarray, W_label_rows: np.ndarray, scale: float) -> float:
    """Error of dH normalised by the maximum of its softmax half.  W_label_rows[i] = W[g_i] (zero
    for a label outside the vocabulary), exact values of the stored weights."""
    soft = dH_ref + scale * W_label_rows
    return float(np.abs(dH_got - dH_ref).max() / max(np.abs(soft).max(), 1e-300))


def dH_softmax_part_bar(dH_ref: np.ndarray, W_label_rows: np.ndarray, scale: float, tol: float, d_is_bf16: bool) -> float:
    """Bar for dH_softmax_part_err.  With D held in bf16 the one-hot element (softmax - 1) * scale is
    rounded with a relative error of up to 2^-9, i.e. an absolute error of 2^-9 * scale * |W[g_i]| in row i
    of dH that does not shrink with V, while the softmax half does: the bar is tol plus that floor
    (doubled).  At large V the floor dominates and this measure only sees gross mistakes; the runs with
    every label outside the vocabulary (G = 0, no such element) are the sharp check of dH there."""
    soft = dH_ref + scale * W_label_rows
    if not d_is_bf16:
        # fp32 end to end: the stated bar (tol of the whole tensor's maximum) expressed relative to the softmax
        # half; with tol = 1e-5 that is sharp as it stands
        return tol * float(np.abs(dH_ref).max()) / max(float(np.abs(soft).max()), 1e-300)
    return tol + 2.0 ** -8 * float(np.abs(W_label_rows).max()) * scale / max(float(np.abs(soft).max()), 1e-300)


def unlabelled_rows(labels: np.ndarray, row_ids: np.ndarray) -> np.ndarray:
    """Mask over row_ids (global vocabulary ids): True where no token of the batch has that label."""
    return ~np.isin(row_ids, labels)


def dW_unlabelled_err(dW_got: np.ndarray, dW_ref: np.ndarray, labels: np.ndarray, row_ids: np.ndarray) -> float:
    """Error over the vocabulary rows without a label, normalised by THOSE rows' maximum.
    dW_got / dW_ref hold the rows listed in row_ids (global ids)."""
    mask = unlabelled_rows(labels, row_ids)
    if not mask.any():
        return 0.0
    ref = dW_ref[mask]
    return float(np.abs(dW_got[mask] - ref).max() / max(np.abs(ref).max(), 1e-300))


def D_elementwise_err(D_got: np.ndarray, D_ref: np.ndarray, atol: float) -> float:
    """max over elements of |got - ref| / (|ref| + atol): a relative error per element, with atol
    keeping elements that underflow towards zero from dominating."""
    return float((np.abs(D_got - D_ref) / (np.abs(D_ref) + atol)).max())


# Bars for the measures above with bf16 operands (D rounded once to bf16, logits rounded to bf16
# when they are stored).  A relative error e per element of D that is independent from element to
# element averages out in the products; what these bars must catch is a systematic error of the
# softmax half - a factor, a dropped term, a wrong statistic - which shows up at its full size.
SOFT_TOL_BF16 = 2e-2          # same number as the stated bar, but relative to the softmax half alone
SOFT_TOL_F32 = 1e-5


def D_rtol_bf16(y_abs_max: float, logits_stored: bool) -> float:
    """Relative tolerance for an element of D in bf16:
    2^-8 for the rounding of D to bf16 (half an ulp is 2^-9, doubled for the one-hot element,
    where softmax - 1 cancels), plus |Y|max * 2^-8 when the logits went through bf16 storage
    (an absolute error of up to |Y| 2^-9 in the exponent, doubled as slack), plus 2e-3 for the fp32
    statistics and the hardware exponential."""
    return 2.0 ** -8 + (y_abs_max * 2.0 ** -8 if logits_stored else 0.0) + 2e-3
