"""GPU parity of the variants beyond Algorithm 1 on equal shards: a short last shard and a
padded vocabulary (the paper pads V to a multiple of 2p), and tied input / output embeddings
(one fp32 gradient buffer per shard receives dW from vp_output_bwd and then the scatter-add of
vp_embed_bwd).  Same bars as the main parity tests; the oracle is the unsharded definition on
the true vocabulary."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import vp_oracle as oc
from gpu_util import GRAD_TOL, LOSS_RTOL, rel_max_err, to_dev, to_host

pytestmark = pytest.mark.gpu


def run_plan(H, Ws, labels, save_logits, vocab_size=None):
    import paper_2411_05288_amd as vp
    plan = vp.driver.OutputLayerPlan(to_dev(H), [to_dev(w) for w in Ws], to_dev(labels), save_logits,
                                     vocab_size=vocab_size)
    plan.workspace.fill_(0xFF)
    plan.step()
    torch.cuda.synchronize()
    return plan


def check_uneven(N, h, rows, V_true, dtype, save_logits, seed):
    total = sum(rows)
    W = si.normal((total, h), 0.08, dtype, seed, si.STREAM_W)
    H = si.normal((N, h), 1.0, dtype, seed, si.STREAM_H)
    labels = si.uniform_ids(N, V_true, seed)
    Ws, off = [], 0
    for n in rows:
        Ws.append(np.ascontiguousarray(W[off:off + n]))
        off += n
    plan = run_plan(H, Ws, labels, save_logits, vocab_size=V_true)
    ref = oc.output_layer(si.as_f64(H), si.as_f64(W[:V_true]), labels)
    tol = GRAD_TOL[dtype]
    loss = float(to_host(plan.loss)[0])
    assert abs(loss - ref["loss"]) <= LOSS_RTOL * abs(ref["loss"])
    assert rel_max_err(to_host(plan.dH).astype(np.float64), ref["dX"]) <= tol
    dW = np.concatenate([to_host(w).astype(np.float64) for w in plan.dW])
    assert rel_max_err(dW[:V_true], ref["dW"]) <= tol
    assert (dW[V_true:] == 0).all(), "padding rows of dW must be zero"
    stat_atol = 2e-3 if dtype == "bf16" else 2e-6 * max(1.0, float(np.abs(ref["Y"]).max()))
    np.testing.assert_allclose(to_host(plan.global_max), ref["m"], rtol=0, atol=stat_atol)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("save_logits", [True, False])
def test_short_last_shard(dtype, save_logits):
    # three shards of 520, 520 and 300 rows: nothing is padding
    check_uneven(200, 128, [520, 520, 300], 1340, dtype, save_logits, seed=41)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("save_logits", [True, False])
def test_vocabulary_padded_to_a_multiple_of_2p(dtype, save_logits):
    # V = 1003, p = 4: padded to 1008 = 4 x 252; the last shard holds 247 real rows and 5 of padding
    check_uneven(150, 64, [252] * 4, 1003, dtype, save_logits, seed=42)


def test_shard_that_is_all_padding():
    # V = 300 on 4 shards of 128 rows: shard 2 has 44 real rows, shard 3 none
    check_uneven(70, 64, [128] * 4, 300, "bf16", True, seed=43)


def test_tied_embeddings_accumulate_into_one_gradient():
    # the output layer's dW_shard and the input layer's table gradient share one fp32 buffer per shard
    import paper_2411_05288_amd as vp
    N, h, V, p = 260, 128, 1024, 2
    Vs = V // p
    H, Ws, labels = si.small_output_case(N, h, V, p, "bf16", seed=51, w_std=0.08)
    ids = si.zipf_ids(N, V, 1.1, 52)
    gout = si.normal((N, h), 1.0, "bf16", 53, si.STREAM_GRAD)
    plan = run_plan(H, Ws, labels, True)              # dW_shard = D^T H (overwrites)
    ws = torch.empty((vp.vp_workspace_bytes(vp.binding.VP_CALL_EMBED_BWD, N, h, Vs, vp.VP_BF16, 0),),
                     dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)
    for r in range(p):                                 # then the embedding gradient adds into it
        vp.vp_embed_bwd(to_dev(gout), to_dev(ids), r * Vs, plan.dW[r], ws)
    torch.cuda.synchronize()
    ref = oc.output_layer(si.as_f64(H), si.as_f64(np.concatenate(Ws)), labels)
    for r in range(p):
        dE = oc.embed_bwd(si.as_f64(gout), ids, r * Vs, Vs, np.zeros((Vs, h)))
        want = ref["dW"][r * Vs:(r + 1) * Vs] + dE
        got = to_host(plan.dW[r]).astype(np.float64)
        # the embedding term is exact in fp32 up to summation rounding; the dW term carries the bf16 bar
        assert np.abs(got - want).max() <= GRAD_TOL["bf16"] * np.abs(ref["dW"]).max() + 1e-5 * np.abs(dE).max()


# ------------------------------------------------------------------ Algorithm 2 (one barrier)
def check_alg2(N, h, V, p, dtype, save_logits, seed, w_std=0.08):
    import paper_2411_05288_amd as vp
    H, Ws, labels = si.small_output_case(N, h, V, p, dtype, seed=seed, w_std=w_std)
    plan = vp.driver.OutputLayerPlan(to_dev(H), [to_dev(w) for w in Ws], to_dev(labels), save_logits, algorithm=2)
    plan.workspace.fill_(0xFF)
    plan.forward()                       # pass S on every shard, the barrier, the input gradient
    torch.cuda.synchronize()
    X, W64 = si.as_f64(H), [si.as_f64(w) for w in Ws]
    ref2 = oc.output_layer_alg2(X, W64, labels)
    full = oc.output_layer(X, np.concatenate(W64), labels)
    tol = GRAD_TOL[dtype]
    # dH is complete after the forward phase: that is the point of Algorithm 2
    assert rel_max_err(to_host(plan.dH).astype(np.float64), full["dX"]) <= tol
    assert rel_max_err(to_host(plan.dH).astype(np.float64), ref2["dX"]) <= tol
    for r in range(p):
        A = to_host(plan.A[r]).astype(np.float64)
        assert rel_max_err(A, ref2["A"][r]) <= tol, "A of shard %d" % r
        Bm = to_host(plan.Bm[r])
        want = si.as_f64(Ws[r])[np.clip(labels - r * (V // p), 0, V // p - 1)]
        own = (labels >= r * (V // p)) & (labels < (r + 1) * (V // p))
        want[~own] = 0.0
        assert np.array_equal(si.as_f64(Bm), want), "B of shard %d is an exact gather" % r
        assert np.array_equal(want, ref2["B"][r])
    loss = float(to_host(plan.loss)[0])
    assert abs(loss - full["loss"]) <= LOSS_RTOL * abs(full["loss"])
    plan.backward()                      # pass T: dW only
    torch.cuda.synchronize()
    dW = np.concatenate([to_host(w).astype(np.float64) for w in plan.dW])
    assert rel_max_err(dW, full["dW"]) <= tol
    assert rel_max_err(dW, np.concatenate(ref2["dW"])) <= tol
    return plan


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("save_logits", [True, False])
@pytest.mark.parametrize("shape", [(300, 136, 1040, 2), (257, 64, 792, 3), (513, 72, 500, 2), (1, 8, 8, 2)])
def test_algorithm2_matches_oracle(shape, save_logits, dtype):
    N, h, V, p = shape
    print("alg2 case", shape, save_logits, dtype, flush=True)
    check_alg2(N, h, V, p, dtype, save_logits, seed=300 + N)


def test_algorithm2_equals_algorithm1_on_the_gpu():
    import paper_2411_05288_amd as vp
    H, Ws, labels = si.small_output_case(520, 256, 2048, 4, "bf16", seed=61, w_std=0.08)
    args = (to_dev(H), [to_dev(w) for w in Ws], to_dev(labels), True)
    a = vp.driver.OutputLayerPlan(*args, algorithm=1)
    b = vp.driver.OutputLayerPlan(*args, algorithm=2)
    a.step()
    b.step()
    torch.cuda.synchronize()
    assert torch.equal(a.loss, b.loss)
    for x, y in zip(a.dW, b.dW):
        assert torch.equal(x, y)         # pass T forms D and dW identically in both algorithms
    # dH: D W (D rounded to bf16) against A c - B (softmax' rounded to bf16): same bar, not the same bits
    assert rel_max_err(to_host(b.dH).astype(np.float64), to_host(a.dH).astype(np.float64)) <= 1e-2


# ------------------------------------------------------------------ barrier on a side stream
def test_barrier_on_a_side_stream_matches_the_serial_order():
    # The paper overlaps its barriers with compute by putting them on separate streams.  Here the barrier's
    # on-device work (vp_combine_stats) runs on a second stream of default priority while a pass-S launch of
    # another microbatch runs on the main stream; both must give bit for bit what the serial order gives.
    import paper_2411_05288_amd as vp
    H, Ws, labels = si.small_output_case(2048, 512, 4096, 2, "bf16", seed=71, w_std=0.05)
    plan = vp.driver.OutputLayerPlan(to_dev(H), [to_dev(w) for w in Ws], to_dev(labels), True)
    plan.forward()
    torch.cuda.synchronize()
    serial = [t.clone() for t in (plan.global_max, plan.global_sumexp, plan.loss_rows, plan.loss,
                                  plan.local_max, plan.local_sumexp, plan.local_target, plan.logits[0])]
    # the barrier reads its own copies of the statistics, the concurrent pass S writes fresh buffers
    lm, ls, lt = plan.local_max.clone(), plan.local_sumexp.clone(), plan.local_target.clone()
    f32 = dict(dtype=torch.float32, device="cuda")
    N = plan.N
    main = torch.cuda.current_stream()
    side = torch.cuda.Stream()          # default priority
    for it in range(4):
        gm, gs, lr, lo = (torch.full((N,), 7.0, **f32), torch.full((N,), 7.0, **f32), torch.full((N,), 7.0, **f32),
                          torch.full((1,), 7.0, **f32))
        m2, s2, t2 = torch.full((N,), 7.0, **f32), torch.full((N,), 7.0, **f32), torch.full((N,), 7.0, **f32)
        y2 = torch.zeros_like(plan.logits[0])
        side.wait_stream(main)
        vp.vp_combine_stats(lm, ls, lt, gm, gs, lr, lo, side)
        vp.vp_output_fwd(plan.H, plan.W[0], plan.labels, 0, m2, s2, t2, y2, plan.workspace)      # main stream
        main.wait_stream(side)
        torch.cuda.synchronize()
        for got, want in zip((gm, gs, lr, lo), serial[:4]):
            assert torch.equal(got, want), "barrier on the side stream differs from the serial order (iteration %d)" % it
        assert torch.equal(m2, serial[4][0]) and torch.equal(s2, serial[5][0]) and torch.equal(t2, serial[6][0])
        assert torch.equal(y2, serial[7])


def test_plan_on_an_explicit_stream_orders_its_own_fills():
    # a plan driven on a stream that is not torch's current one: the torch-side fills (padding rows of dW,
    # the neutral statistics of an all-padding shard) must be ordered with the library's kernels on that stream
    import paper_2411_05288_amd as vp
    H = si.normal((70, 64), 1.0, "bf16", 43, si.STREAM_H)
    W = si.normal((512, 64), 0.08, "bf16", 43, si.STREAM_W)
    labels = si.uniform_ids(70, 300, 43)
    Ws = [np.ascontiguousarray(W[r * 128:(r + 1) * 128]) for r in range(4)]
    ref = oc.output_layer(si.as_f64(H), si.as_f64(W[:300]), labels)
    for algorithm in (1, 2):
        plan = vp.driver.OutputLayerPlan(to_dev(H), [to_dev(w) for w in Ws], to_dev(labels), True, vocab_size=300,
                                         algorithm=algorithm)
        for w in plan.dW:
            w.fill_(5.0)
        plan.dH.fill_(5.0)
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        plan.step(side)
        side.synchronize()
        dW = np.concatenate([to_host(w).astype(np.float64) for w in plan.dW])
        assert rel_max_err(dW[:300], ref["dW"]) <= GRAD_TOL["bf16"] and (dW[300:] == 0).all()
        assert rel_max_err(to_host(plan.dH).astype(np.float64), ref["dX"]) <= GRAD_TOL["bf16"]
        assert abs(float(to_host(plan.loss)[0]) - ref["loss"]) <= LOSS_RTOL * abs(ref["loss"])
