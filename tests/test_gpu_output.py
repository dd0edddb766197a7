"""Parity of the HIP output-layer path (vp_output_fwd / vp_combine_stats / vp_output_bwd,
called through the C ABI) against the CPU oracle on the same seeded inputs.

Bars: loss within relative 1e-3; dH and dW within 2e-2 * max|tensor| for bf16 inputs and
1e-5 * max|tensor| for fp32 inputs (max-abs error); statistics compared with tolerances
derived from fp32 accumulation of K <= 8192 products (|dY| <~ 1e-4 at |Y| ~ 5)."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import vp_oracle as oc
from gpu_util import GRAD_TOL, LOSS_RTOL, rel_max_err, run_output_layer, to_dev, to_host, to_host_f64

pytestmark = pytest.mark.gpu


def check_against_oracle(H, Ws, labels, save_logits, grad_scale=None, tag="", grad_tol=None):
    dtype = "bf16" if H.dtype == np.uint16 else "f32"
    plan = run_output_layer(H, Ws, labels, save_logits, grad_scale)
    X = si.as_f64(H)
    W64 = [si.as_f64(w) for w in Ws]
    ref = oc.output_layer_alg1(X, W64, labels, grad_scale)
    full = oc.output_layer(X, np.concatenate(W64), labels, grad_scale)   # the unsharded definition

    # absolute error of a logit grows with its magnitude (fp32 accumulation)
    ymax = max(1.0, float(np.abs(full["Y"]).max()))
    stat_atol = (2e-3 if dtype == "bf16" else 2e-6) * ymax
    stat_rtol = 2e-3 if dtype == "bf16" else 2e-5 * ymax
    np.testing.assert_allclose(to_host(plan.local_max), ref["m_loc"], rtol=0, atol=stat_atol, err_msg=tag)
    np.testing.assert_allclose(to_host(plan.local_sumexp), ref["sum_loc"], rtol=stat_rtol, err_msg=tag)
    np.testing.assert_allclose(to_host(plan.local_target), ref["t_loc"], rtol=0, atol=stat_atol, err_msg=tag)
    np.testing.assert_allclose(to_host(plan.global_max), full["m"], rtol=0, atol=stat_atol, err_msg=tag)
    np.testing.assert_allclose(to_host(plan.global_sumexp), full["sum"], rtol=stat_rtol, err_msg=tag)
    np.testing.assert_allclose(to_host(plan.loss_rows), full["loss_rows"], rtol=LOSS_RTOL, atol=stat_atol, err_msg=tag)
    loss = float(to_host(plan.loss)[0])
    assert abs(loss - full["loss"]) <= LOSS_RTOL * abs(full["loss"]), tag
    if save_logits:
        for r in range(len(Ws)):
            y = to_host_f64(plan.logits[r])
            ytol = (2.0 ** -8) * np.abs(ref["Y"][r]).max() + 1e-6 if dtype == "bf16" else stat_atol
            np.testing.assert_allclose(y, ref["Y"][r], rtol=0, atol=ytol, err_msg=tag)
    tol = GRAD_TOL[dtype] if grad_tol is None else grad_tol
    e_dH = rel_max_err(to_host(plan.dH).astype(np.float64), full["dX"])
    assert e_dH <= tol, "%s dH err %g" % (tag, e_dH)
    dW = np.concatenate([to_host(w).astype(np.float64) for w in plan.dW])
    e_dW = rel_max_err(dW, full["dW"])
    assert e_dW <= tol, "%s dW err %g" % (tag, e_dW)
    for r in range(len(Ws)):     # every shard against Algorithm 1 run on the CPU
        assert np.abs(to_host(plan.dW[r]) - ref["dW"][r]).max() <= tol * np.abs(full["dW"]).max(), tag
    return {"loss_rel": abs(loss - full["loss"]) / abs(full["loss"]), "dH": e_dH, "dW": e_dW}


# shapes chosen to span several 256x256 tiles with ragged tails in every dimension, a K that
# is not a multiple of the 64-wide K step, and sizes that break 16-byte row alignment
SMALL = [
    # N,   h,   V,    p
    (300, 136, 1040, 2),     # Vs = 520 = 2 tiles + 8 columns; K tail of 8
    (257, 64, 792, 3),       # Vs = 264; N one row past a tile
    (64, 200, 512, 1),       # single shard (textbook cross-entropy)
    (513, 72, 500, 2),       # Vs = 250: rows of D not 16-byte aligned
    (130, 100, 520, 2),      # h = 100: rows of H and W not 16-byte aligned
    (1, 8, 8, 2),            # degenerate: one token, 4 vocabulary rows per shard
]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("save_logits", [True, False])
@pytest.mark.parametrize("shape", SMALL)
def test_small_cases_match_oracle(shape, save_logits, dtype):
    N, h, V, p = shape
    H, Ws, labels = si.small_output_case(N, h, V, p, dtype, seed=101 + N, w_std=0.08)
    print("case", shape, save_logits, dtype, flush=True)
    check_against_oracle(H, Ws, labels, save_logits, tag=str((shape, save_logits, dtype)))


def test_cfg1_tiny_fp32():
    cfg = si.CONFIGS["cfg1_tiny"]
    H = si.make_H(cfg)
    Ws = [si.make_W_shard(cfg, r) for r in range(cfg.p)]
    labels = si.make_labels(cfg)
    err = check_against_oracle(H, Ws, labels, cfg.save_logits, tag="cfg1")
    print("cfg1 errors", err, flush=True)


def test_unscaled_gradients_and_large_logits():
    # grad_scale = 1 is the paper's unscaled form; W scaled so that |Y| reaches ~150,
    # where an unshifted exp would overflow fp32
    H, Ws, labels = si.small_output_case(96, 64, 768, 3, "f32", seed=5, w_std=5.0)
    ymax = float(np.abs(si.as_f64(H) @ si.as_f64(np.concatenate(Ws)).T).max())
    assert ymax > 100
    # Derived bar.  An fp32 logit of magnitude |Y| carries an absolute error eps of a few ulp(|Y|); to first
    # order a perturbation of the logits of a row by at most eps changes softmax_j by at most 2 eps softmax_j
    # (d softmax_j = softmax_j (dY_j - sum_k softmax_k dY_k)), hence dH and dW by at most 2 eps of their
    # magnitude.  With eps = 2 ulp_fp32(|Y|max) that is 4 ulp on top of the 1e-5 of the benign configurations
    # (ulp(150) = 1.5e-5: about 7e-5 here; 1.1e-5 is what the kernels achieve).
    grad_tol = 1e-5 + 4.0 * float(np.spacing(np.float32(ymax)))
    check_against_oracle(H, Ws, labels, True, grad_scale=1.0, tag="large-logits f32", grad_tol=grad_tol)
    H, Ws, labels = si.small_output_case(96, 64, 768, 3, "bf16", seed=5, w_std=2.0)
    plan = run_output_layer(H, Ws, labels, False, 1.0)
    assert np.isfinite(to_host(plan.dH)).all() and np.isfinite(to_host(plan.loss)).all()


def test_labels_outside_every_shard_are_not_owned():
    # ids outside [0, V) belong to no shard: target 0 on every shard, all-zero one-hot row
    N, h, V, p = 70, 64, 512, 2
    H, Ws, labels = si.small_output_case(N, h, V, p, "bf16", seed=9)
    labels = labels.copy()
    labels[::3] = V + 5
    labels[1::7] = -3
    plan = run_output_layer(H, Ws, labels, True)
    X, W64 = si.as_f64(H), [si.as_f64(w) for w in Ws]
    ref = oc.output_layer_alg1(X, W64, labels)       # the oracle's one_hot uses the same rule
    np.testing.assert_allclose(to_host(plan.local_target), ref["t_loc"], atol=2e-3)
    assert (to_host(plan.local_target)[:, ::3] == 0).all()
    assert rel_max_err(to_host(plan.dH).astype(np.float64), ref["dX"]) <= 2e-2
    dW = np.concatenate([to_host(w).astype(np.float64) for w in plan.dW])
    assert rel_max_err(dW, np.concatenate(ref["dW"])) <= 2e-2


def test_runs_are_bitwise_repeatable_and_dH_accumulates():
    H, Ws, labels = si.small_output_case(300, 128, 1024, 2, "bf16", seed=77)
    a = run_output_layer(H, Ws, labels, True)
    b = run_output_layer(H, Ws, labels, True)
    for x, y in [(a.dH, b.dH), (a.loss, b.loss), (a.local_sumexp, b.local_sumexp), (a.dW[1], b.dW[1])]:
        assert torch.equal(x, y)
    # dH_accum is accumulate-into: a second backward without zeroing doubles it
    import paper_2411_05288_amd as vp
    first = a.dH.clone()
    for r in range(a.p):
        vp.vp_output_bwd(a.H, a.W[r], a.labels, r * a.Vs, a.global_max, a.global_sumexp, a.logits[r],
                         a.grad_scale, a.dH, a.dW[r], a.workspace)
    torch.cuda.synchronize()
    np.testing.assert_allclose(to_host(a.dH), 2 * to_host(first), rtol=1e-6, atol=1e-9)


def test_stored_and_recomputed_logits_agree():
    H, Ws, labels = si.small_output_case(260, 192, 1536, 2, "bf16", seed=31)
    a = run_output_layer(H, Ws, labels, True)
    b = run_output_layer(H, Ws, labels, False)
    assert torch.equal(a.loss, b.loss)
    # the stored path rounds Y to bf16 once more than the recomputing path
    assert rel_max_err(to_host(a.dH).astype(np.float64), to_host(b.dH).astype(np.float64)) < 1e-2


def test_generic_gemm_kernel_on_aligned_shapes():
    # aligned shapes normally take the fast kernel; the generic one must give the same answers
    import paper_2411_05288_amd as vp
    vp.vp_profile_force_generic_gemm(True)
    try:
        H, Ws, labels = si.small_output_case(300, 128, 1040, 2, "bf16", seed=3, w_std=0.08)
        check_against_oracle(H, Ws, labels, True, tag="generic kernel, stored logits")
        check_against_oracle(H, Ws, labels, False, tag="generic kernel, recompute")
    finally:
        vp.vp_profile_force_generic_gemm(False)


def test_step_can_be_captured_in_a_hip_graph():
    # the library allocates nothing, synchronises nothing and records no memset: a whole step can be
    # captured once and replayed.  Every replay is checked against the eager result, with eager work
    # and synchronisations between the replays.
    import paper_2411_05288_amd as vp
    H, Ws, labels = si.small_output_case(300, 136, 1040, 2, "bf16", seed=17, w_std=0.08)
    plan = vp.driver.OutputLayerPlan(to_dev(H), [to_dev(w) for w in Ws], to_dev(labels), True)
    plan.step()
    torch.cuda.synchronize()
    want = [plan.loss.clone(), plan.dH.clone(), plan.dW[0].clone(), plan.dW[1].clone(), plan.local_sumexp.clone()]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        plan.step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        plan.step()
    torch.cuda.synchronize()
    for i in range(4):
        plan.dH.fill_(3.0)
        plan.loss.zero_()
        plan.dW[1].fill_(-1.0)
        plan.workspace.fill_(0xFF)
        g.replay()
        torch.cuda.synchronize()
        got = [plan.loss, plan.dH, plan.dW[0], plan.dW[1], plan.local_sumexp]
        for a, b in zip(got, want):
            assert torch.equal(a, b), "replay %d differs from the eager step" % i
        plan.step()                      # eager work between replays
        torch.cuda.synchronize()


def _random_shapes(seed, count):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        p = int(rng.integers(1, 5))
        Vs = int(rng.choice([int(rng.integers(1, 40)), int(rng.integers(40, 700)), 8 * int(rng.integers(1, 90))]))
        h = int(rng.choice([int(rng.integers(1, 50)), 8 * int(rng.integers(1, 40)), 64 * int(rng.integers(1, 6))]))
        N = int(rng.choice([int(rng.integers(1, 20)), int(rng.integers(20, 600))]))
        out.append((N, h, Vs * p, p))
    return out


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_random_shapes_match_oracle(dtype):
    # seeded draw of shapes: odd sizes, sizes below one tile, aligned and unaligned rows, both logits modes
    for k, (N, h, V, p) in enumerate(_random_shapes(20241105, 14)):
        H, Ws, labels = si.small_output_case(N, h, V, p, dtype, seed=900 + k, w_std=0.08)
        for save_logits in (True, False):
            print("random case", (N, h, V, p), save_logits, dtype, flush=True)
            check_against_oracle(H, Ws, labels, save_logits, tag=str((N, h, V, p, save_logits, dtype)))


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_more_than_65535_token_rows(dtype):
    # kernels that carry the token row in grid.y work in slabs of 65535 rows; Vs = 12 keeps the
    # elementwise D kernel on its scalar path, which is the one that slabs
    H, Ws, labels = si.small_output_case(70000, 16, 24, 2, dtype, seed=71, w_std=0.2)
    for save_logits in (True, False):
        check_against_oracle(H, Ws, labels, save_logits, tag="70000 rows %s %s" % (dtype, save_logits))


def _guarded(shape, dtype, fill, guard=4096):
    """A contiguous tensor of `shape` cut from the middle of a larger buffer filled with `fill`."""
    n = int(np.prod(shape))
    big = torch.full((n + 2 * guard,), fill, dtype=dtype, device="cuda")
    return big, big[guard:guard + n].view(*shape), guard


@pytest.mark.parametrize("shape", [
    # N,   h,   Vs:  every output tile is ragged in rows and columns
    (300, 128, 1000),     # 16-byte aligned rows everywhere: the descriptor-bounded store path
    (257, 64, 264),       # one row past a row tile, 8 columns past a column tile
    (513, 72, 250),       # rows of the logits / D not 16-byte aligned: the element-wise store path
])
@pytest.mark.parametrize("save_logits", [True, False])
def test_nothing_is_written_outside_the_output_extents(shape, save_logits):
    # the GEMM epilogues store through descriptors sized to the tile's rows and rely on the hardware
    # dropping what lies beyond; every output sits between guard bands that must keep their fill,
    # and so must the workspace beyond the size the library asks for
    import paper_2411_05288_amd as vp
    N, h, Vs = shape
    H, Ws, labels = si.small_output_case(N, h, Vs, 1, "bf16", seed=91)
    Hd, Wd, ld = to_dev(H), to_dev(Ws[0]), to_dev(labels)
    f32, bf16 = torch.float32, torch.bfloat16
    flags = vp.VP_SAVE_LOGITS if save_logits else 0
    need = max(vp.vp_workspace_bytes(vp.binding.VP_CALL_OUTPUT_FWD, N, h, Vs, vp.VP_BF16, flags),
               vp.vp_workspace_bytes(vp.binding.VP_CALL_OUTPUT_BWD, N, h, Vs, vp.VP_BF16, flags), 256)
    ws_big = torch.full((need + 8192,), 0x5A, dtype=torch.uint8, device="cuda")
    bufs = {}
    for name, shp, dt, fill in [("lm", (N,), f32, 7.0), ("ls", (N,), f32, 7.0), ("lt", (N,), f32, 7.0),
                                ("logits", (N, Vs), bf16, 7.0), ("dH", (N, h), f32, 7.0), ("dW", (Vs, h), f32, 7.0)]:
        bufs[name] = _guarded(shp, dt, fill)
    t = {k: v[1] for k, v in bufs.items()}
    vp.vp_output_fwd(Hd, Wd, ld, 0, t["lm"], t["ls"], t["lt"], t["logits"] if save_logits else None, ws_big[:need])
    t["dH"].zero_()
    vp.vp_output_bwd(Hd, Wd, ld, 0, t["lm"].clone(), t["ls"].clone(), t["logits"] if save_logits else None, 1.0 / N,
                     t["dH"], t["dW"], ws_big[:need])
    torch.cuda.synchronize()
    for name, (big, view, guard) in bufs.items():
        assert bool((big[:guard] == 7.0).all()) and bool((big[guard + view.numel():] == 7.0).all()), \
            "%s: written outside its extent" % name
    assert bool((ws_big[need:] == 0x5A).all()), "workspace written beyond the size vp_workspace_bytes returned"
    # and what is inside is right: one shard, so the local statistics are the global ones
    ref = oc.output_layer(si.as_f64(H), si.as_f64(Ws[0]), labels)
    assert rel_max_err(to_host(t["dH"]).astype(np.float64), ref["dX"]) <= GRAD_TOL["bf16"]
    assert rel_max_err(to_host(t["dW"]).astype(np.float64), ref["dW"]) <= GRAD_TOL["bf16"]
    if save_logits:
        y = to_host_f64(t["logits"])
        assert np.abs(y - ref["Y"]).max() <= (2.0 ** -8) * np.abs(ref["Y"]).max() + 1e-6
