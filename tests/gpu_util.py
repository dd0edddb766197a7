"""Helpers for the GPU parity tests: move seeded NumPy inputs to the GPU, run the HIP path
through the C-ABI binding, bring results back as NumPy."""
from __future__ import annotations

import numpy as np
import torch

import synth_inputs as si


def to_dev(x: np.ndarray) -> torch.Tensor:
    """uint16 arrays are bf16 bit patterns; everything else keeps its dtype."""
    if x.dtype == np.uint16:
        return torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(x).cuda()


def to_host(t: torch.Tensor) -> np.ndarray:
    """Back to NumPy; bf16 comes back as uint16 bit patterns."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def to_host_f64(t: torch.Tensor) -> np.ndarray:
    return si.as_f64(to_host(t))


def run_output_layer(H, Ws, labels, save_logits=True, grad_scale=None):
    import paper_2411_05288_amd as vp
    plan = vp.driver.OutputLayerPlan(to_dev(H), [to_dev(w) for w in Ws], to_dev(labels), save_logits, grad_scale)
    # workspace contents are undefined on entry: poison it (0xFFFF is a bf16 NaN, 0xFFFFFFFF an fp32 NaN) so
    # that any read of scratch the library did not write first (e.g. the row padding of D) shows up
    plan.workspace.fill_(0xFF)
    plan.step()
    torch.cuda.synchronize()
    return plan


# tolerances of the parity bar
LOSS_RTOL = 1e-3          # stated bar for the loss (the tests also report the achieved error)
GRAD_TOL = {"bf16": 2e-2, "f32": 1e-5}   # max-abs error / max|tensor|


def rel_max_err(got: np.ndarray, ref: np.ndarray) -> float:
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-300))


def run_output_layer_keep_D(H, Ws, labels, save_logits=True, grad_scale=None):
    """The same step with pass T called shard by shard through the binding, reading the D matrix that
    vp_output_bwd leaves at the start of its workspace after every shard.  Returns (plan, [D_r]) with
    D_r the [N, Vs_r] values as fp64 (row padding checked to be zero and cut off)."""
    import paper_2411_05288_amd as vp
    plan = vp.driver.OutputLayerPlan(to_dev(H), [to_dev(w) for w in Ws], to_dev(labels), save_logits, grad_scale)
    plan.workspace.fill_(0xFF)
    plan.forward()
    Ds = []
    N = plan.N
    for r in range(plan.p):
        Vs = plan.rows[r]
        vp.vp_output_bwd(plan.H, plan.W[r], plan.labels, plan.offsets[r], plan.global_max, plan.global_sumexp,
                         plan.logits[r] if plan.logits is not None else None, plan.grad_scale,
                         plan.dH, plan.dW[r], plan.workspace, dh_overwrite=(r == 0))
        torch.cuda.synchronize()
        ld = vp.vp_dlogits_row_stride(Vs, plan.dt)
        tdt = torch.float32 if plan.dt == vp.VP_F32 else torch.bfloat16
        esz = 4 if plan.dt == vp.VP_F32 else 2
        D = plan.workspace[:N * ld * esz].view(tdt).view(N, ld)
        full = to_host_f64(D)
        assert (full[:, Vs:] == 0).all(), "row padding of D must be zero"
        Ds.append(np.ascontiguousarray(full[:, :Vs]))
    return plan, Ds
