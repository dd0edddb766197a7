"""Parity at the full sizes of the benchmark configurations, in the launch configuration
bench.py times (same plan, same entry points, same flags).

The oracle evaluates the logits and the row statistics of every token over the whole vocabulary
in fp64 (stats_streamed), then, shard by shard, the definition of D (D_block) and the products
dH += D W_r and dW_r = D^T X.  What is compared:

  cfg2, cfg3  every element of: statistics, loss rows, stored logits, D of every shard, dH, dW.
  cfg4        every element of: statistics, loss rows, D of every shard (formed by the recompute
              GEMM's epilogue), dH; dW on 32 sampled rows of every block of 256 vocabulary rows of
              every shard (one eighth of dW; every output tile of the dW kernel is looked at, and a
              full fp64 dW would be 17 TFLOP more on the host).

Bars: the stated ones (loss 1e-3, dH / dW 2e-2 of the tensor maximum), and - because that maximum is
set by the one-hot half of D - the measures of parity_metrics.py that see the softmax half: D element
by element, the dW rows without a label against their own maximum, and a second step in which every
label lies outside the vocabulary (G = 0), where dH and dW are the softmax half alone and the stated
bar applies to it.  On top, regression bars at about five times the errors these kernels achieve."""
import time

import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import vp_oracle as oc
import parity_metrics as pm
from gpu_util import GRAD_TOL, LOSS_RTOL, to_dev, to_host, to_host_f64

pytestmark = pytest.mark.gpu

# Regression guards, tighter than the stated bars: about five times what these kernels achieve where that
# leaves room (achieved at cfg2 / cfg3: loss 3e-8 / 9e-8, dH 6.6e-4 / 3.6e-4, dW 4.6e-4 / 2.0e-5), about twice
# for the softmax-half measures, which sit nearer their bar because logits stored in bf16 carry a relative
# error of up to |Y| 2^-9 ~ 1.4 % into single elements of D (achieved: D 1.96e-2 of a bar of 3.5e-2, dW rows
# without a label 0.9e-2 / 1.2e-2, G = 0 step dH 5.8e-3 / 2.6e-3 and dW 6.6e-3 / 6.9e-3).
REGRESSION = {
    "loss_rel": 1e-6, "D": 3e-2, "dH": 3e-3, "dW": 2e-3, "dW_unlabelled": 2e-2, "dH_G0": 1.5e-2, "dW_G0": 1.5e-2,
}


def _bwd_shard(vp, plan, r):
    vp.vp_output_bwd(plan.H, plan.W[r], plan.labels, plan.offsets[r], plan.global_max, plan.global_sumexp,
                     plan.logits[r] if plan.logits is not None else None, plan.grad_scale,
                     plan.dH, plan.dW[r], plan.workspace, dh_overwrite=(r == 0))
    torch.cuda.synchronize()


def _read_D(vp, plan, r):
    N, Vs = plan.N, plan.rows[r]
    ld = vp.vp_dlogits_row_stride(Vs, plan.dt)
    full = to_host_f64(plan.workspace[:N * ld * 2].view(torch.bfloat16).view(N, ld))
    assert (full[:, Vs:] == 0).all(), "row padding of D must be zero"
    return full[:, :Vs]


def _sample_rows(Vs, per_tile, rng):
    return np.sort(np.concatenate([b + rng.choice(min(256, Vs - b), min(per_tile, Vs - b), replace=False)
                                   for b in range(0, Vs, 256)]))


def _full_size_check(cfg, dW_rows_per_tile=None):
    """dW_rows_per_tile None: all of dW; else that many sampled rows of every 256-row tile of every shard."""
    import paper_2411_05288_amd as vp
    N, Vs, p, V = cfg.N, cfg.Vs, cfg.p, cfg.V
    scale = 1.0 / N
    tol = GRAD_TOL["bf16"]
    H = si.make_H(cfg)
    labels = si.make_labels(cfg)
    Ws = [si.make_W_shard(cfg, r) for r in range(cfg.p)]
    X = si.as_f64(H)
    plan = vp.driver.OutputLayerPlan(to_dev(H), [to_dev(w) for w in Ws], to_dev(labels), cfg.save_logits)
    plan.workspace.fill_(0xFF)
    rng = np.random.default_rng(12345)
    errs = {}

    t0 = time.time()
    st = oc.stats_streamed(X, (si.as_f64(w) for w in Ws), labels)
    print("%s oracle logits + statistics: %.1f s" % (cfg.name, time.time() - t0), flush=True)
    ymax = max(float(np.abs(y).max()) for y in st["Y"])

    for labelled in (True, False):
        tag = cfg.name + ("" if labelled else " G=0")
        lab = labels if labelled else np.where(np.arange(N) % 2 == 0, V + 11, -1).astype(np.int64)
        plan.labels = to_dev(lab)
        plan.forward()
        torch.cuda.synchronize()
        if labelled:
            # pass S and the barrier: every row
            np.testing.assert_allclose(to_host(plan.global_max), st["m"], rtol=0, atol=2e-3)
            np.testing.assert_allclose(to_host(plan.global_sumexp), st["sum"], rtol=2e-3)
            np.testing.assert_allclose(to_host(plan.loss_rows), st["loss_rows"], rtol=LOSS_RTOL, atol=2e-3)
            loss = float(to_host(plan.loss)[0])
            errs["loss_rel"] = abs(loss - st["loss"]) / abs(st["loss"])
            assert errs["loss_rel"] <= LOSS_RTOL
            if cfg.save_logits:
                for r in range(p):
                    y = to_host_f64(plan.logits[r])
                    assert np.abs(y - st["Y"][r]).max() <= 2.0 ** -8 * ymax + 1e-6, "stored logits of shard %d" % r
        # pass T shard by shard
        t0 = time.time()
        dH_ref = np.zeros((N, cfg.h))
        eD = 0.0
        dW_err = dW_max = unl_err = unl_max = 0.0
        colsum = np.zeros(cfg.h)
        for r in range(p):
            _bwd_shard(vp, plan, r)
            D_ref = oc.D_block(st["Y"][r], st["m"], st["sum"], lab, r * Vs, scale)
            eD = max(eD, pm.D_elementwise_err(_read_D(vp, plan, r), D_ref, atol=1e-9 * scale))
            dH_ref += D_ref @ si.as_f64(Ws[r])
            rows = np.arange(Vs) if (dW_rows_per_tile is None and labelled) else _sample_rows(
                Vs, dW_rows_per_tile or 32, rng)
            dW_ref = D_ref[:, rows].T @ X
            dW_got = plan.dW[r][torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
            dW_err = max(dW_err, float(np.abs(dW_got - dW_ref).max()))
            dW_max = max(dW_max, float(np.abs(dW_ref).max()), float(plan.dW[r].abs().max()) if len(rows) < Vs else 0.0)
            unl = pm.unlabelled_rows(lab, r * Vs + rows)
            if unl.any():
                unl_err = max(unl_err, float(np.abs(dW_got[unl] - dW_ref[unl]).max()))
                unl_max = max(unl_max, float(np.abs(dW_ref[unl]).max()))
            colsum += plan.dW[r].double().sum(dim=0).cpu().numpy()
        print("%s oracle D, dH, dW: %.1f s" % (tag, time.time() - t0), flush=True)
        dH = to_host(plan.dH).astype(np.float64)
        e_dH = pm.rel_max_err(dH, dH_ref)
        e_dW = dW_err / dW_max
        e_unl = unl_err / max(unl_max, 1e-300)
        rtolD = pm.D_rtol_bf16(ymax, cfg.save_logits)
        print("%s: D elem %.3g (bar %.3g)  dH %.3g  dW %.3g  dW unlabelled rows %.3g" % (tag, eD, rtolD, e_dH, e_dW, e_unl),
              flush=True)
        assert eD <= rtolD, tag
        assert e_dH <= tol and e_dW <= tol and e_unl <= tol, tag
        # a property that holds at any size: every column of the full dW sums to scale * sum_i (1 - [g_i in V]) X_i
        want = scale * X[~((lab >= 0) & (lab < V))].sum(axis=0)
        # (the sum over V rows is compared at the bar of the larger of the two scales involved)
        assert np.abs(colsum - want).max() <= 2e-2 * max(float(np.abs(want).max()), 4 * dW_max), tag
        if labelled:
            errs.update({"D": eD, "dH": e_dH, "dW": e_dW, "dW_unlabelled": e_unl})
        else:
            errs.update({"D": max(errs["D"], eD), "dH_G0": e_dH, "dW_G0": e_dW})
    print("%s achieved: %s" % (cfg.name, {k: float("%.3g" % v) for k, v in errs.items()}), flush=True)
    for k, bar in REGRESSION.items():
        assert errs[k] <= bar, "%s: %s regressed to %.3g (guard %.3g)" % (cfg.name, k, errs[k], bar)


@pytest.mark.timeout(900)
def test_cfg2_llama_every_element():
    _full_size_check(si.CONFIGS["cfg2_llama"])


@pytest.mark.timeout(900)
def test_cfg3_large_vocab_every_element():
    _full_size_check(si.CONFIGS["cfg3_large_vocab"])


@pytest.mark.timeout(1100)
def test_cfg4_very_large_vocab_recompute_dW_sampled():
    _full_size_check(si.CONFIGS["cfg4_very_large_vocab"], dW_rows_per_tile=32)
