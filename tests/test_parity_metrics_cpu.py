"""Which error measure can see a mistake in the softmax half of D?  CPU only: the mistakes are
planted in the oracle's D (section 4.2: D = (softmax - G) / N), never in the HIP path.

For each planted mistake the gradients are formed from the wrong D with the oracle's own
products and compared with the right ones.  The whole-tensor measure of the stated parity bar
stays under 2e-2 for dW at these sizes (the one-hot rows set the maximum), while the measures
that take the one-hot half out (tests/parity_metrics.py) exceed their bars by a wide margin -
so the GPU tests, which apply both, cannot pass with such a mistake in a kernel."""
import functools

import numpy as np
import pytest

import synth_inputs as si
from oracle import vp_oracle as oc
import parity_metrics as pm

# (name, factor on the softmax half): dropped entirely, 20 % low, 30 % high
MISTAKES = [("dropped", 0.0), ("scaled_0.8", 0.8), ("scaled_1.3", 1.3)]


@functools.lru_cache(maxsize=None)
def _case(labels_kind):
    N, h, V, p = 512, 64, 16384, 2
    H, Ws, labels = si.small_output_case(N, h, V, p, "bf16", seed=23, labels=labels_kind, w_std=0.02)
    X = si.as_f64(H)
    W = np.concatenate([si.as_f64(w) for w in Ws])
    ref = oc.output_layer(X, W, labels)
    return X, W, labels, ref


@pytest.mark.parametrize("labels_kind", ["uniform", "zipf"])
@pytest.mark.parametrize("name,factor", MISTAKES)
def test_planted_softmax_mistakes_are_seen_only_by_the_new_measures(labels_kind, name, factor):
    X, W, labels, ref = _case(labels_kind)
    N, V = X.shape[0], W.shape[0]
    scale = 1.0 / N
    P = oc.softmax(ref["Y"])
    D_bad = (factor * P - oc.one_hot(labels, V)) * scale
    dH_bad, dW_bad = D_bad @ W, D_bad.T @ X

    # the stated bar's measure on dW does not see it
    assert pm.rel_max_err(dW_bad, ref["dW"]) < 2e-2, "whole-tensor dW measure unexpectedly sharp"
    # the measures with the one-hot half taken out do
    rows = np.arange(V)
    e_dW = pm.dW_unlabelled_err(dW_bad, ref["dW"], labels, rows)
    e_dH = pm.dH_softmax_part_err(dH_bad, ref["dX"], W[labels], scale)
    e_D = pm.D_elementwise_err(D_bad, ref["D"], atol=1e-9 * scale)
    want = abs(1.0 - factor)
    assert e_dW == pytest.approx(want, rel=1e-6)
    assert e_dH == pytest.approx(want, rel=1e-6)
    assert e_D >= 0.9 * want
    assert e_dW > 5 * pm.SOFT_TOL_BF16
    # dH with labels present: the bar has to allow for the bf16 rounding of the one-hot element of D, a
    # floor of about 0.2 of the softmax half at this V, so this measure only sees the gross mistake ...
    if factor == 0.0:
        assert e_dH > 1.5 * pm.dH_softmax_part_bar(ref["dX"], W[labels], scale, pm.SOFT_TOL_BF16, d_is_bf16=True)
    # ... and the sharp check of dH is the run below
    # every label outside the vocabulary (G = 0): the stated whole-tensor measure is then sharp for both
    nolab_labels = np.full_like(labels, V + 7)
    nolab = oc.output_layer_alg1(X, [W], nolab_labels)     # (the sharded form accepts labels nobody owns)
    Dn_bad = factor * P * scale
    assert pm.rel_max_err(Dn_bad @ W, nolab["dX"]) == pytest.approx(want, rel=1e-6)
    assert pm.rel_max_err(Dn_bad.T @ X, nolab["dW"][0]) == pytest.approx(want, rel=1e-6)
    assert e_D > 5 * pm.D_rtol_bf16(float(np.abs(ref["Y"]).max()), logits_stored=True)


def test_measures_vanish_for_the_right_D_and_for_bf16_rounding_of_it():
    # the right D gives zero; D rounded to bf16 (what the kernels feed the products) stays far below the bars
    X, W, labels, ref = _case("uniform")
    N, V = X.shape[0], W.shape[0]
    scale = 1.0 / N
    rows = np.arange(V)
    assert pm.dW_unlabelled_err(ref["dW"], ref["dW"], labels, rows) == 0.0
    assert pm.dH_softmax_part_err(ref["dX"], ref["dX"], W[labels], scale) == 0.0
    D16 = si.as_f64(si.f32_to_bf16_bits(ref["D"].astype(np.float32)))
    assert pm.D_elementwise_err(D16, ref["D"], atol=1e-9 * scale) <= 2.0 ** -8
    e_dW = pm.dW_unlabelled_err(D16.T @ X, ref["dW"], labels, rows)
    e_dH = pm.dH_softmax_part_err(D16 @ W, ref["dX"], W[labels], scale)
    assert e_dW < pm.SOFT_TOL_BF16 / 5
    # dH carries the rounding of the one-hot element of D, which the derived bar allows for
    bar = pm.dH_softmax_part_bar(ref["dX"], W[labels], scale, pm.SOFT_TOL_BF16, d_is_bf16=True)
    assert e_dH < bar / 2 and bar < 0.5
    # without labels in the vocabulary there is no such element and dH is sharp at the plain bar
    nolab = oc.output_layer_alg1(X, [W], np.full_like(labels, V + 7))
    D16n = si.as_f64(si.f32_to_bf16_bits(nolab["D"][0].astype(np.float32)))
    assert pm.rel_max_err(D16n @ W, nolab["dX"]) < pm.SOFT_TOL_BF16 / 5


def test_labels_outside_the_vocabulary_leave_only_the_softmax_half():
    # with every label outside [0, V) the one-hot matrix is zero and the whole-tensor measure is the
    # softmax-half measure: the device used by the GPU tests to aim the stated bar at the softmax term
    X, W, labels, _ = _case("uniform")
    V = W.shape[0]
    out = oc.output_layer_alg1(X, [W[: V // 2], W[V // 2:]], np.full_like(labels, V + 7))
    assert all(np.all(oc.one_hot(np.full_like(labels, V + 7), V // 2, off) == 0) for off in (0, V // 2))
    colsum = np.concatenate(out["D"], axis=1).sum(axis=1)
    np.testing.assert_allclose(colsum, 1.0 / X.shape[0], rtol=1e-12)   # rows of D sum to scale * 1
