"""Parity of the HIP input-layer path (vp_embed_fwd / vp_embed_bwd through the C ABI) against
the CPU oracle.  The gather must be bit exact.  The scatter-add adds duplicate ids in
increasing token position starting from the accumulator's value, the same order as the
oracle's fp32 loop, so it is compared bit for bit with that loop and, within 1e-6 * max, with
the fp64 result."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import vp_oracle as oc
from gpu_util import to_dev, to_host

pytestmark = pytest.mark.gpu


def run_embed(tables, ids, gout, dtable0=None):
    import paper_2411_05288_amd as vp
    plan = vp.driver.EmbeddingPlan([to_dev(t) for t in tables], to_dev(ids), to_dev(gout))
    if dtable0 is not None:
        for d, d0 in zip(plan.dtable, dtable0):
            d.copy_(to_dev(d0))
    plan.workspace.fill_(0xFF)       # scratch contents are undefined on entry
    plan.forward()
    plan.backward()
    torch.cuda.synchronize()
    return plan


def check_embed(N, h, V, p, dtype, seed, ids=None, preload=False):
    Vs = V // p
    tables = [si.normal((Vs, h), 0.02, dtype, seed, si.STREAM_TABLE, r) for r in range(p)]
    gout = si.normal((N, h), 1.0, dtype, seed, si.STREAM_GRAD)
    if ids is None:
        ids = si.zipf_ids(N, V, 1.1, seed)
    d0 = [si.normal((Vs, h), 0.5, "f32", seed, 9, r) for r in range(p)] if preload else None
    plan = run_embed(tables, ids, gout, d0)
    g32 = si.as_f32(gout)
    for r in range(p):
        out_ref = oc.embed_fwd(tables[r], ids, r * Vs)
        assert np.array_equal(to_host(plan.out[r]), out_ref), "gather shard %d" % r
        base32 = d0[r].copy() if preload else np.zeros((Vs, h), dtype=np.float32)
        ref32 = oc.embed_bwd(g32, ids, r * Vs, Vs, base32)
        ref64 = oc.embed_bwd(g32.astype(np.float64), ids, r * Vs, Vs,
                             (d0[r].astype(np.float64) if preload else np.zeros((Vs, h))))
        got = to_host(plan.dtable[r])
        assert np.array_equal(got, ref32), "scatter-add shard %d differs from the in-order fp32 sum" % r
        assert np.abs(got - ref64).max() <= 1e-6 * max(np.abs(ref64).max(), 1e-30) * 8
    return plan


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("shape", [
    (700, 256, 4096, 4),     # several ids per row, Zipf duplicates
    (33, 40, 64, 2),         # row bytes 80 (bf16): 16-byte vectors; tiny vocabulary: long runs
    (129, 36, 96, 3),        # bf16 rows of 72 bytes: not a multiple of 16 -> scalar path
    (1, 8, 16, 2),
    (20000, 64, 5000, 2),    # more keys than one sorting workgroup holds (multi-chunk sort)
    (8192, 200, 32, 2),      # the one-kernel path at its largest N; runs far longer than a workgroup's chunk; ragged slab
    (3000, 37, 64, 2),       # odd row length: one column per lane
])
def test_embed_small_cases(shape, dtype):
    N, h, V, p = shape
    print("embed case", shape, dtype, flush=True)
    check_embed(N, h, V, p, dtype, seed=200 + N)


def test_embed_accumulates_into_existing_gradient():
    check_embed(300, 128, 1024, 2, "bf16", seed=3, preload=True)


def test_embed_ids_outside_vocabulary_and_all_out_of_shard():
    N, h, V, p = 64, 64, 256, 2
    ids = si.uniform_ids(N, V, 5)
    ids[::5] = V + 100
    ids[1::9] = -1
    check_embed(N, h, V, p, "bf16", seed=5, ids=ids)
    # every id lives in shard 0: shard 1 must produce zeros and leave its gradient untouched
    ids = si.uniform_ids(N, V // 2, 6)
    plan = check_embed(N, h, V, p, "bf16", seed=6, ids=ids)
    assert float(plan.out[1].float().abs().max()) == 0.0 and float(plan.dtable[1].abs().max()) == 0.0


def test_embed_bwd_bitwise_repeatable():
    a = check_embed(2000, 128, 512, 2, "bf16", seed=8)
    b = check_embed(2000, 128, 512, 2, "bf16", seed=8)
    for x, y in zip(a.dtable, b.dtable):
        assert torch.equal(x, y)


@pytest.mark.timeout(600)
def test_cfg5_embedding_full_size():
    cfg = si.CONFIGS["cfg5_embedding"]
    tables = [si.make_table_shard(cfg, r) for r in range(cfg.p)]
    ids = si.make_labels(cfg)
    gout = si.make_grad_out(cfg)
    plan = run_embed(tables, ids, gout)
    g32 = si.as_f32(gout)
    total = np.zeros((cfg.N, cfg.h), dtype=np.float32)
    for r in range(cfg.p):
        out = to_host(plan.out[r])
        assert np.array_equal(out, oc.embed_fwd(tables[r], ids, r * cfg.Vs))
        total += si.bf16_bits_to_f32(out)
        ref32 = oc.embed_bwd(g32, ids, r * cfg.Vs, cfg.Vs, np.zeros((cfg.Vs, cfg.h), dtype=np.float32))
        got = to_host(plan.dtable[r])
        assert np.array_equal(got, ref32)
        own = (ids >= r * cfg.Vs) & (ids < (r + 1) * cfg.Vs)
        ref_colsum = g32[own].astype(np.float64).sum(axis=0)
        np.testing.assert_allclose(got.astype(np.float64).sum(axis=0), ref_colsum, rtol=0,
                                   atol=1e-4 * max(np.abs(ref_colsum).max(), 1.0))
    # the sum over shards is the plain lookup
    full_table = np.concatenate(tables)
    assert np.array_equal(total, si.bf16_bits_to_f32(full_table[ids]))


def test_embed_key_packing_limits():
    # the one-kernel path packs (row, token) into 32 bits: 13 bits of token, 2^19 - 1 rows per shard; one row more
    # per shard takes the general path.  (N * Vs < 2^31 is the library's limit, hence N = 4000 here.)
    N, h = 4000, 8
    for Vs in (2 ** 19 - 1, 2 ** 19):
        ids = si.uniform_ids(N, 2 * Vs, 31)
        ids[-1] = Vs - 1
        ids[-2] = 2 * Vs - 1
        ids[:40] = Vs - 1          # and a long run on that row
        print("embed key limits Vs", Vs, flush=True)
        check_embed(N, h, 2 * Vs, 2, "bf16", seed=31, ids=ids)


def test_embed_more_than_65535_tokens():
    # N above the grid.y limit and above one sorting chunk; tiny vocabulary: very long runs of equal ids
    check_embed(70000, 8, 48, 2, "bf16", seed=72)
