"""Parity of the D matrix itself (row a4: D = (softmax - G) * scale, Algorithm 1 pass T with the
rescale identity of section 4.3 folded in) and of the softmax half of dH and dW.

The whole-tensor bar on dH / dW is dominated by the one-hot half of D (see parity_metrics.py), so
this file adds what can see the other half:
  * D read back from the workspace after vp_output_bwd and compared element by element with the
    oracle, for stored and for recomputed logits (the elementwise kernel and the GEMM epilogue);
  * runs in which every label lies outside the vocabulary, so that G = 0 and dH, dW consist of the
    softmax half alone: the stated bar then applies to exactly that half;
  * the vocabulary rows of dW that carry no label, normalised by their own maximum.
Bars: stated ones (2e-2 bf16 / 1e-5 fp32) on the softmax half; per element of D the tolerance
derived in parity_metrics.D_rtol_bf16 (bf16) or from fp32 rounding of the logits (fp32)."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import vp_oracle as oc
import parity_metrics as pm
from gpu_util import GRAD_TOL, run_output_layer_keep_D, to_host

pytestmark = pytest.mark.gpu


def check_D_and_softmax_half(H, Ws, labels, save_logits, tag, grad_scale=None):
    dtype = "bf16" if H.dtype == np.uint16 else "f32"
    plan, Ds = run_output_layer_keep_D(H, Ws, labels, save_logits, grad_scale)
    X = si.as_f64(H)
    W64 = [si.as_f64(w) for w in Ws]
    ref = oc.output_layer_alg1(X, W64, labels, grad_scale)
    N = X.shape[0]
    scale = plan.grad_scale
    ymax = max(1.0, max(float(np.abs(y).max()) for y in ref["Y"]))
    if dtype == "bf16":
        rtol = pm.D_rtol_bf16(ymax, save_logits)
    else:
        # fp32 logits carry an absolute error of a few ulp of |Y|max into the exponent
        rtol = 8 * np.finfo(np.float32).eps * ymax + 1e-5
    worst = 0.0
    for r in range(len(Ws)):
        e = pm.D_elementwise_err(Ds[r], ref["D"][r], atol=1e-9 * scale)
        worst = max(worst, e)
        assert e <= rtol, "%s shard %d: D element error %.3g > %.3g" % (tag, r, e, rtol)
        # the one-hot elements are where D changes sign: they must be negative and close to -scale
        loc = labels - plan.offsets[r]
        own = (loc >= 0) & (loc < Ws[r].shape[0])
        if own.any():
            got = Ds[r][np.nonzero(own)[0], loc[own]]
            assert (got < 0).all(), tag
    # rows of D over the whole vocabulary sum to scale * (1 - [label in the vocabulary])
    rowsum = sum(d.sum(axis=1) for d in Ds)
    V = sum(w.shape[0] for w in Ws)
    want = scale * (1.0 - ((labels >= 0) & (labels < V)))
    np.testing.assert_allclose(rowsum, want, rtol=0, atol=(rtol + 2.0 ** -8) * scale, err_msg=tag)

    tol = GRAD_TOL[dtype]
    dH = to_host(plan.dH).astype(np.float64)
    dW = np.concatenate([to_host(w).astype(np.float64) for w in plan.dW])
    dW_ref = np.concatenate(ref["dW"])
    Wfull = np.concatenate(W64)
    in_vocab = (labels >= 0) & (labels < V)
    W_lab = np.where(in_vocab[:, None], Wfull[np.clip(labels, 0, V - 1)], 0.0)
    e_soft_dH = pm.dH_softmax_part_err(dH, ref["dX"], W_lab, scale)
    bar_dH = pm.dH_softmax_part_bar(ref["dX"], W_lab, scale, tol, d_is_bf16=(dtype == "bf16"))
    e_unl_dW = pm.dW_unlabelled_err(dW, dW_ref, labels, np.arange(V))
    print("%s: D elem %.3g (bar %.3g)  dH soft %.3g (bar %.3g)  dW unlabelled %.3g (bar %.3g)  dH %.3g dW %.3g" % (
        tag, worst, rtol, e_soft_dH, bar_dH, e_unl_dW, tol, pm.rel_max_err(dH, ref["dX"]), pm.rel_max_err(dW, dW_ref)),
        flush=True)
    assert e_soft_dH <= bar_dH, tag
    assert e_unl_dW <= tol, tag
    assert pm.rel_max_err(dH, ref["dX"]) <= tol and pm.rel_max_err(dW, dW_ref) <= tol, tag
    return {"D": worst, "dH_soft": e_soft_dH, "dW_unl": e_unl_dW}


SHAPES = [
    # N,   h,   V,    p
    (300, 136, 1040, 2),     # ragged tiles, K tail
    (257, 64, 792, 3),
    (513, 72, 500, 2),       # rows of D not 16-byte aligned: element-wise store path
    (600, 256, 4096, 2),     # several tiles per product
    (1, 8, 8, 2),
]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("save_logits", [True, False])
@pytest.mark.parametrize("shape", SHAPES)
def test_D_matches_the_definition_element_by_element(shape, save_logits, dtype):
    N, h, V, p = shape
    H, Ws, labels = si.small_output_case(N, h, V, p, dtype, seed=301 + N, w_std=0.08)
    check_D_and_softmax_half(H, Ws, labels, save_logits, "D %s stored=%s %s" % (shape, save_logits, dtype))


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("save_logits", [True, False])
@pytest.mark.parametrize("shape", SHAPES[:4])
def test_no_label_in_the_vocabulary_softmax_half_alone(shape, save_logits, dtype):
    # G = 0: dH and dW are the softmax half and the stated whole-tensor bar applies to it directly
    N, h, V, p = shape
    H, Ws, labels = si.small_output_case(N, h, V, p, dtype, seed=401 + N, w_std=0.08)
    labels = np.where(np.arange(N) % 2 == 0, V + 5, -3).astype(np.int64)
    check_D_and_softmax_half(H, Ws, labels, save_logits, "G=0 %s stored=%s %s" % (shape, save_logits, dtype))


def test_unscaled_form_and_zipf_labels():
    # grad_scale = 1 (the paper's unscaled gradients) and a skewed label distribution: many tokens share a label
    H, Ws, labels = si.small_output_case(700, 128, 2048, 4, "bf16", seed=55, labels="zipf", w_std=0.08)
    check_D_and_softmax_half(H, Ws, labels, True, "zipf stored scale=1", grad_scale=1.0)
    check_D_and_softmax_half(H, Ws, labels, False, "zipf recompute scale=1", grad_scale=1.0)
