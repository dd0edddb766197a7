"""Pins for the CPU oracle: it is checked against what the paper's equations and plain
mathematics fix (closed forms, identities, finite differences, brute force), never
against itself and never against the HIP path.  The paper prints no numeric example
for the vocabulary layers, so there is no printed value to compare with."""
import math

import numpy as np
import pytest

import synth_inputs as si
from oracle import vp_oracle as oc


def _case(N=6, h=5, V=12, p=3, seed=3, w_std=0.3):
    H, Ws, labels = si.small_output_case(N, h, V, p, "f32", seed=seed, w_std=w_std)
    return si.as_f64(H), [si.as_f64(w) for w in Ws], labels


# ----------------------------------------------------------------------------- loss
def test_loss_matches_naive_unshifted_form():
    # -ln( e^{Y_ig} / sum_j e^{Y_ij} ) written with Python floats and no max shift
    X, Ws, g = _case()
    W = np.concatenate(Ws)
    ref = oc.output_layer(X, W, g)
    for i in range(X.shape[0]):
        y = [sum(X[i, k] * W[j, k] for k in range(X.shape[1])) for j in range(W.shape[0])]
        naive = -math.log(math.exp(y[g[i]]) / sum(math.exp(v) for v in y))
        assert abs(naive - ref["loss_rows"][i]) < 1e-12


def test_loss_closed_form_zero_weights_and_zero_hidden():
    X, Ws, g = _case(N=7, h=4, V=20, p=4)
    W = np.concatenate(Ws)
    assert oc.output_layer(X, np.zeros_like(W), g)["loss"] == pytest.approx(math.log(20), abs=1e-14)
    assert oc.output_layer(np.zeros_like(X), W, g)["loss"] == pytest.approx(math.log(20), abs=1e-14)
    out = oc.output_layer_alg1(np.zeros_like(X), Ws, g)
    assert out["loss"] == pytest.approx(math.log(20), abs=1e-14)


@pytest.mark.parametrize("p", [1, 2, 4, 8, 16])
def test_sharded_equals_unsharded_for_every_p(p):
    N, h, V = 9, 7, 64
    H, Ws, g = si.small_output_case(N, h, V, p, "f32", seed=11, w_std=0.5)
    X = si.as_f64(H)
    Ws = [si.as_f64(w) for w in Ws]
    W = np.concatenate(Ws)
    ref = oc.output_layer(X, W, g)
    a1 = oc.output_layer_alg1(X, Ws, g)
    a2 = oc.output_layer_alg2(X, Ws, g)
    np.testing.assert_allclose(a1["loss_rows"], ref["loss_rows"], rtol=0, atol=1e-13)
    np.testing.assert_allclose(a1["m"], ref["m"], rtol=0, atol=0)
    np.testing.assert_allclose(a1["sum"], ref["sum"], rtol=1e-14)
    np.testing.assert_allclose(a1["dX"], ref["dX"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(np.concatenate(a1["dW"]), ref["dW"], rtol=0, atol=1e-15)
    # Algorithm 2's identity for the input gradient (section 4.4) gives the same result
    np.testing.assert_allclose(a2["dX"], ref["dX"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(np.concatenate(a2["dW"]), ref["dW"], rtol=0, atol=1e-15)


def test_large_logits_do_not_overflow_and_match_high_precision():
    # |Y| around 200: a naive fp32 exp overflows; the shifted form must agree with an
    # evaluation done with Python's arbitrary-precision-safe log-sum-exp via math.fsum
    X, Ws, g = _case(N=5, h=6, V=16, p=4, w_std=40.0)
    W = np.concatenate(Ws)
    ref = oc.output_layer(X, W, g)
    assert np.abs(ref["Y"]).max() > 150
    with np.errstate(over="ignore"):
        assert np.isinf(np.exp(ref["Y"].astype(np.float32)).max())   # the naive fp32 route breaks
    a1 = oc.output_layer_alg1(X, Ws, g)
    for i in range(5):
        y = ref["Y"][i]
        big = y.max()
        lse = big + math.log(math.fsum(math.exp(v - big) for v in y))
        assert ref["loss_rows"][i] == pytest.approx(lse - y[g[i]], rel=1e-13)
        assert a1["loss_rows"][i] == pytest.approx(lse - y[g[i]], rel=1e-13)
    assert np.isfinite(a1["dX"]).all() and np.isfinite(np.concatenate(a1["dW"])).all()


def test_vocabulary_permutation_invariance():
    X, Ws, g = _case(N=8, h=5, V=24, p=2)
    W = np.concatenate(Ws)
    perm = np.random.default_rng(0).permutation(24)      # new row j holds old row perm[j]
    inv = np.argsort(perm)
    a = oc.output_layer(X, W, g)
    b = oc.output_layer(X, W[perm], inv[g])
    np.testing.assert_allclose(a["loss_rows"], b["loss_rows"], atol=1e-13)
    np.testing.assert_allclose(a["dX"], b["dX"], atol=1e-15)
    np.testing.assert_allclose(a["dW"][perm], b["dW"], atol=1e-15)


# ------------------------------------------------------------------- softmax and D
def test_softmax_rows_sum_to_one_across_shards_and_rescale_identity():
    X, Ws, g = _case(N=10, h=6, V=48, p=4, w_std=1.5)
    W = np.concatenate(Ws)
    a1 = oc.output_layer_alg1(X, Ws, g, grad_scale=1.0)
    full = np.concatenate(a1["softmax"], axis=1)
    np.testing.assert_allclose(full.sum(axis=1), 1.0, atol=1e-14)
    # element-wise: softmax' * sum' e^{m'-m} / sum  ==  direct softmax of the full row
    np.testing.assert_allclose(full, oc.softmax(oc.logits(X, W)), atol=1e-15)
    D = np.concatenate(a1["D"], axis=1)
    np.testing.assert_allclose(D.sum(axis=1), 0.0, atol=1e-14)
    # using the un-rescaled local sum instead would break the row sums
    S = [oc.alg1_S(X, w, g, 12 * r) for r, w in enumerate(Ws)]
    m, resc, s = oc.alg1_C1([q["m_loc"] for q in S], [q["sum_loc"] for q in S])
    wrong = np.concatenate([S[r]["softmax_loc"] * (S[r]["sum_loc"] / s)[:, None] for r in range(4)], axis=1)
    assert np.abs(wrong.sum(axis=1) - 1.0).max() > 1e-3


def test_combine_is_associative_and_identity_on_one_shard():
    rng = np.random.default_rng(5)
    m = rng.normal(size=(6, 9)) * 4
    s = rng.uniform(1, 50, size=(6, 9))
    t = np.zeros((6, 9))
    allm, _, alls = oc.alg1_C1(m, s)
    # fold 0..2 and 3..5 separately, then fold the two results
    ma, _, sa = oc.alg1_C1(m[:3], s[:3])
    mb, _, sb = oc.alg1_C1(m[3:], s[3:])
    m2, _, s2 = oc.alg1_C1([ma, mb], [sa, sb])
    np.testing.assert_array_equal(m2, allm)
    np.testing.assert_allclose(s2, alls, rtol=1e-14)
    order = rng.permutation(6)
    m3, _, s3 = oc.alg1_C1(m[order], s[order])
    np.testing.assert_array_equal(m3, allm)
    np.testing.assert_allclose(s3, alls, rtol=1e-14)
    m1, _, s1 = oc.alg1_C1(m[:1], s[:1])
    np.testing.assert_array_equal(m1, m[0])
    np.testing.assert_array_equal(s1, s[0])
    # closed form: log-sum-exp of the pieces
    lse = np.log((s * np.exp(m)).sum(axis=0))
    np.testing.assert_allclose(oc.combine_stats(m, s, t)["loss_rows"], lse, rtol=1e-13)


# ------------------------------------------------------------------------ gradients
def _loss_only(X, W, g):
    return oc.output_layer(X, W, g)["loss"]


def test_gradients_match_central_finite_differences():
    N, h, V, p = 4, 5, 12, 3
    X, Ws, g = _case(N=N, h=h, V=V, p=p, w_std=0.7)
    W = np.concatenate(Ws)
    out = oc.output_layer_alg1(X, Ws, g)
    dW = np.concatenate(out["dW"])
    eps = 1e-6
    for i in range(N):
        for k in range(h):
            Xp, Xm = X.copy(), X.copy()
            Xp[i, k] += eps
            Xm[i, k] -= eps
            fd = (_loss_only(Xp, W, g) - _loss_only(Xm, W, g)) / (2 * eps)
            assert abs(fd - out["dX"][i, k]) < 1e-7
    for j in range(V):
        for k in range(h):
            Wp, Wm = W.copy(), W.copy()
            Wp[j, k] += eps
            Wm[j, k] -= eps
            fd = (_loss_only(X, Wp, g) - _loss_only(X, Wm, g)) / (2 * eps)
            assert abs(fd - dW[j, k]) < 1e-7


def test_gradient_closed_forms():
    N, h, V = 6, 4, 10
    X, Ws, g = _case(N=N, h=h, V=V, p=2)
    W = np.concatenate(Ws)
    # W = 0: softmax is uniform -> dX = 0, dW_j = (1/N) sum_i (1/V - [g_i = j]) X_i
    o = oc.output_layer_alg1(X, [np.zeros_like(w) for w in Ws], g)
    np.testing.assert_allclose(o["dX"], 0.0, atol=1e-16)
    exp_dW = np.zeros((V, h))
    for i in range(N):
        for j in range(V):
            exp_dW[j] += (1.0 / V - (1.0 if g[i] == j else 0.0)) * X[i] / N
    np.testing.assert_allclose(np.concatenate(o["dW"]), exp_dW, atol=1e-15)
    # H = 0: dW = 0, dX_i = (1/N)(mean_j W_j - W_{g_i})
    o = oc.output_layer_alg1(np.zeros_like(X), Ws, g)
    np.testing.assert_allclose(np.concatenate(o["dW"]), 0.0, atol=1e-16)
    exp_dX = np.stack([(W.mean(axis=0) - W[g[i]]) / N for i in range(N)])
    np.testing.assert_allclose(o["dX"], exp_dX, atol=1e-15)


def test_dW_column_sums_vanish_and_grad_scale_is_linear():
    X, Ws, g = _case(N=12, h=6, V=40, p=5, w_std=1.0)
    o1 = oc.output_layer_alg1(X, Ws, g)                 # 1/N
    np.testing.assert_allclose(np.concatenate(o1["dW"]).sum(axis=0), 0.0, atol=1e-14)
    o2 = oc.output_layer_alg1(X, Ws, g, grad_scale=1.0)  # the paper's unscaled form
    np.testing.assert_allclose(o2["dX"], o1["dX"] * 12, rtol=1e-13, atol=1e-16)


def test_alg2_A_B_terms():
    # A*sum'/sum - B summed over shards is N times the mean-loss input gradient
    X, Ws, g = _case(N=5, h=4, V=18, p=3, w_std=1.2)
    a2 = oc.output_layer_alg2(X, Ws, g, grad_scale=1.0)
    ref = oc.output_layer(X, np.concatenate(Ws), g)
    np.testing.assert_allclose(a2["dX"], ref["dX"] * 5, atol=1e-14)
    # B is the gathered label row on the owning shard, zero elsewhere
    W = np.concatenate(Ws)
    np.testing.assert_allclose(sum(a2["B"]), W[g], atol=0)


def test_streamed_stats_and_blocks_equal_full():
    X, Ws, g = _case(N=9, h=5, V=30, p=3, w_std=1.1)
    ref = oc.output_layer(X, np.concatenate(Ws), g)
    st = oc.stats_streamed(X, iter(Ws), g)
    np.testing.assert_array_equal(st["m"], ref["m"])
    np.testing.assert_allclose(st["sum"], ref["sum"], rtol=1e-14)
    np.testing.assert_allclose(st["loss_rows"], ref["loss_rows"], atol=1e-13)
    D = np.concatenate([oc.D_block(st["Y"][r], st["m"], st["sum"], g, 10 * r, 1.0 / 9) for r in range(3)], axis=1)
    np.testing.assert_allclose(D, ref["D"], atol=1e-16)


# ------------------------------------------------------------------------ embedding
def test_embed_fwd_sum_over_shards_is_full_lookup_bit_exact():
    V, h, N, p = 40, 8, 33, 4
    table = si.normal((V, h), 0.02, "bf16", 1, si.STREAM_TABLE)
    ids = si.zipf_ids(N, V, 1.1, 2)
    total = np.zeros((N, h), dtype=np.float32)
    for r in range(p):
        out = oc.embed_fwd(table[r * 10:(r + 1) * 10], ids, r * 10)
        own = (ids >= r * 10) & (ids < (r + 1) * 10)
        assert (out[~own] == 0).all()                       # +0 bit pattern
        np.testing.assert_array_equal(out[own], table[ids[own]])
        total += si.bf16_bits_to_f32(out)
    np.testing.assert_array_equal(total, si.bf16_bits_to_f32(table[ids]))


def test_embed_bwd_equals_dense_one_hot_product():
    V, h, N, p = 24, 6, 50, 3
    Vs = V // p
    g = si.as_f64(si.normal((N, h), 1.0, "bf16", 4, si.STREAM_GRAD))
    ids = si.zipf_ids(N, V, 1.1, 9)
    for r in range(p):
        dE = oc.embed_bwd(g, ids, r * Vs, Vs, np.zeros((Vs, h)))
        onehot = oc.one_hot(ids, Vs, r * Vs)                # [N, Vs]
        np.testing.assert_allclose(dE, onehot.T @ g, atol=1e-13)
        own = (ids >= r * Vs) & (ids < (r + 1) * Vs)
        assert (np.abs(dE).sum(axis=1) > 0).sum() == len(np.unique(ids[own]))
        np.testing.assert_allclose(dE.sum(axis=0), g[own].sum(axis=0), atol=1e-12)
    # accumulate-into: a second call adds on top of the first
    dE = oc.embed_bwd(g, ids, 0, Vs, np.zeros((Vs, h)))
    dE2 = oc.embed_bwd(g, ids, 0, Vs, dE.copy())
    np.testing.assert_allclose(dE2, 2 * dE, atol=1e-13)
    # fp32 accumulation in token order stays within rounding of the fp64 result
    dE32 = oc.embed_bwd(g.astype(np.float32), ids, 0, Vs, np.zeros((Vs, h), dtype=np.float32))
    np.testing.assert_allclose(dE32, dE, rtol=0, atol=1e-5 * np.abs(dE).max())


# ------------------------------------------------------------------ input generators
def test_bf16_round_trip_and_rounding():
    x = np.array([1.0, 1.00390625, 1.005859375, -2.5, 3.0e-3, 0.0], dtype=np.float32)
    b = si.f32_to_bf16_bits(x)
    back = si.bf16_bits_to_f32(b)
    assert back[0] == 1.0 and back[3] == -2.5 and back[5] == 0.0
    assert back[1] == 1.0            # 1 + 2^-8 is a tie: rounds to even (1.0)
    assert back[2] == 1.0078125      # 1 + 1.5*2^-8 rounds up to 1 + 2^-7
    assert np.abs(back - x).max() <= np.abs(x).max() * 2 ** -8
    y = si.normal((1000,), 1.0, "bf16", 1, 1)
    assert si.f32_to_bf16_bits(si.bf16_bits_to_f32(y)).tolist() == y.tolist()


def test_zipf_structure():
    ids = si.zipf_ids(8192, 256000, 1.1, si.BASE_SEED)
    assert ids.min() >= 0 and ids.max() < 256000
    _, counts = np.unique(ids, return_counts=True)
    # the hottest id takes roughly 1/H_{V,1.1} ~ 13 % of the tokens
    assert 0.09 < counts.max() / 8192 < 0.17
    assert 2000 < len(counts) < 4500
    assert (si.zipf_ids(8192, 256000, 1.1, si.BASE_SEED) == ids).all()


def test_oracle_matches_its_stored_tiny_case():
    # tests/golden/oracle_tiny_case.json is written by tests/golden/make_oracle_golden.py (oracle only);
    # it guards the oracle's arithmetic against silent change
    import importlib.util
    import json
    import os
    here = os.path.dirname(os.path.abspath(__file__))
    spec = importlib.util.spec_from_file_location("make_oracle_golden", os.path.join(here, "golden", "make_oracle_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    now = mod.compute()
    stored = json.load(open(os.path.join(here, "golden", "oracle_tiny_case.json")))
    assert now["labels"] == stored["labels"] and now["ids"] == stored["ids"]
    for k in ("loss", "m", "sum", "m_loc", "sum_loc", "dX", "dW_shard1", "alg2_dX", "alg2_A0", "embed_bwd_shard1"):
        np.testing.assert_allclose(np.asarray(now[k]), np.asarray(stored[k]), rtol=1e-12, atol=1e-15, err_msg=k)
