"""Element-by-element parity on shapes that reach the code paths the benchmark configurations run
at full size, with a small contraction length so that the oracle stays cheap:

  * more output tiles than compute units: persistent workgroups walking several tiles, outputs
    written with streaming stores (every product of cfg3 / cfg4);
  * at most 16 tile rows with several rounds (the forward and dH products: contiguous runs per XCD);
  * more than 16 tile rows (the dW products: tiles ranked in 16 x 16 blocks), also with 17 and more
    tile columns, so that blocks are clipped at both edges of the grid;
  * ragged last tiles in both directions on top of that.

Everything the path produces is compared with the oracle: stored logits, statistics, loss, D, dH
and dW, with the stated bars plus the measures of parity_metrics.py that see the softmax half."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import vp_oracle as oc
import parity_metrics as pm
from gpu_util import GRAD_TOL, LOSS_RTOL, run_output_layer_keep_D, to_dev, to_host, to_host_f64

pytestmark = pytest.mark.gpu

TILE = 256
CUS = 256


def tiles(m, n):
    return -(-m // TILE), -(-n // TILE)


def full_check(N, h, Vs, p, save_logits, seed, labels_kind="uniform"):
    V = Vs * p
    H, Ws, labels = si.small_output_case(N, h, V, p, "bf16", seed=seed, labels=labels_kind, w_std=0.02)
    plan, Ds = run_output_layer_keep_D(H, Ws, labels, save_logits)
    X = si.as_f64(H)
    W64 = [si.as_f64(w) for w in Ws]
    ref = oc.output_layer_alg1(X, W64, labels)
    scale = 1.0 / N
    ymax = max(1.0, max(float(np.abs(y).max()) for y in ref["Y"]))
    # statistics and loss
    np.testing.assert_allclose(to_host(plan.local_max), ref["m_loc"], rtol=0, atol=2e-3 * ymax)
    np.testing.assert_allclose(to_host(plan.local_sumexp), ref["sum_loc"], rtol=2e-3)
    np.testing.assert_allclose(to_host(plan.local_target), ref["t_loc"], rtol=0, atol=2e-3 * ymax)
    loss = float(to_host(plan.loss)[0])
    assert abs(loss - ref["loss"]) <= LOSS_RTOL * abs(ref["loss"])
    # stored logits, every element
    if save_logits:
        for r in range(p):
            y = to_host_f64(plan.logits[r])
            assert np.abs(y - ref["Y"][r]).max() <= 2.0 ** -8 * ymax + 1e-6, "stored logits, shard %d" % r
    # D, every element
    rtol = pm.D_rtol_bf16(ymax, save_logits)
    eD = max(pm.D_elementwise_err(Ds[r], ref["D"][r], atol=1e-9 * scale) for r in range(p))
    assert eD <= rtol, "D element error %.3g > %.3g" % (eD, rtol)
    # gradients, every element: the stated bar and the softmax-half measures
    tol = GRAD_TOL["bf16"]
    dH = to_host(plan.dH).astype(np.float64)
    dW = np.concatenate([to_host(w).astype(np.float64) for w in plan.dW])
    dW_ref = np.concatenate(ref["dW"])
    e_dH, e_dW = pm.rel_max_err(dH, ref["dX"]), pm.rel_max_err(dW, dW_ref)
    e_unl = pm.dW_unlabelled_err(dW, dW_ref, labels, np.arange(V))
    Wfull = np.concatenate(W64)
    e_soft = pm.dH_softmax_part_err(dH, ref["dX"], Wfull[labels], scale)
    bar_soft = pm.dH_softmax_part_bar(ref["dX"], Wfull[labels], scale, tol, True)
    print("N=%d h=%d Vs=%d p=%d stored=%s: D %.3g dH %.3g dW %.3g dW-unlabelled %.3g dH-soft %.3g (bar %.3g)" % (
        N, h, Vs, p, save_logits, eD, e_dH, e_dW, e_unl, e_soft, bar_soft), flush=True)
    assert e_dH <= tol and e_dW <= tol and e_unl <= tol and e_soft <= bar_soft
    return plan


@pytest.mark.timeout(600)
@pytest.mark.parametrize("save_logits", [True, False])
def test_more_tiles_than_compute_units_17_tile_rows(save_logits):
    # forward 17 x 17 = 289 tiles, dH 17 x 16 = 272, dW 17 x 16 = 272: all persistent multi-tile with streaming
    # stores, all with more than 16 tile rows (16 x 16 block order, clipped blocks)
    N, h, Vs = 4352, 4096, 4352
    for m, n in [(N, Vs), (N, h), (Vs, h)]:
        tm, tn = tiles(m, n)
        assert tm * tn > CUS and tm > 16
    full_check(N, h, Vs, 1, save_logits, seed=611)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("save_logits", [True, False])
def test_more_tiles_than_compute_units_16_tile_rows_17_tile_columns(save_logits):
    # forward 16 x 17 and dH 16 x 17 tiles (at most 16 tile rows: contiguous runs per XCD, two rounds),
    # dW 17 x 17 (block order with 17 tile columns); two shards, so dH also takes the accumulating epilogue
    N, h, Vs = 4096, 4352, 4352
    (tm, tn) = tiles(N, Vs)
    assert tm == 16 and tn == 17
    assert tiles(N, h) == (16, 17) and tiles(Vs, h) == (17, 17)
    full_check(N, h, Vs, 2, save_logits, seed=612, labels_kind="zipf")


@pytest.mark.timeout(600)
@pytest.mark.parametrize("save_logits", [True, False])
def test_more_tiles_than_compute_units_ragged_edges(save_logits):
    # the same with ragged last tiles in every direction: N = 16 * 256 + 4, h = 16 * 256 + 64, Vs = 17 * 256 + 8
    N, h, Vs = 4100, 4160, 4360
    for m, n in [(N, Vs), (N, h), (Vs, h)]:
        tm, tn = tiles(m, n)
        assert tm * tn > CUS and tm > 16
    full_check(N, h, Vs, 1, save_logits, seed=613)


def test_the_shapes_above_run_the_persistent_fast_kernel():
    # the kernel's own timeline header says how many workgroups and tiles the traced launch had
    import paper_2411_05288_amd as vp
    N, h, Vs = 4352, 4096, 4352
    H, Ws, labels = si.small_output_case(N, h, Vs, 1, "bf16", seed=611, w_std=0.02)
    plan = vp.driver.OutputLayerPlan(to_dev(H), [to_dev(w) for w in Ws], to_dev(labels), True)
    buf = torch.zeros(8 + 256 * 4 * 8, dtype=torch.int64, device="cuda")
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    for name, want_tiles in [("gemm_bf16_fwd_stats", 17 * 17), ("gemm_bf16_dH", 17 * 16), ("gemm_bf16_dW", 17 * 16)]:
        buf.zero_()
        vp.vp_profile_gemm_trace(buf, name)
        try:
            plan.step()
            torch.cuda.synchronize()
        finally:
            vp.vp_profile_gemm_trace(None)
        head = buf[:3].cpu().numpy()
        assert head[1] == want_tiles, (name, head)
        assert head[0] == min(cus, want_tiles) and head[2] == -(-want_tiles // head[0]), (name, head)
        if want_tiles > cus:
            assert head[2] >= 2      # at least one workgroup walked two tiles
